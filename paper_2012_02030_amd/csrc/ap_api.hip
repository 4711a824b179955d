// C ABI of the library: host-side validation and dispatch.  See include/ap.h for the contract.
#include <hip/hip_runtime.h>
#include <initializer_list>
#include <math.h>
#include <mutex>
#include <stdint.h>

#include "ap.h"
#include "ap_internal.h"

namespace {

inline bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Scratch of ap_sparse_attn_fwd_split_static: partial outputs and their log-sum-exp.  Part of the
// code object, so every GPU that loads the library holds its own copy at its own address.  In
// host code the name is only a handle for hipGetSymbolAddress; the kernels get the address.
static __device__ __align__(256) unsigned char scratch[AP_FWD_SPLIT_STATIC_MAX_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};      // per device, resolved on the first call there

// Address of the current device's copy of `scratch` (null on failure).
void* static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

bool strides_ok(const int64_t* s, int D, int elems_per_16b)
{
    for (int k = 0; k < 3; ++k)
        if (s[k] < 0 || s[k] % elems_per_16b != 0) return false;
    return s[2] >= D;
}

}  // namespace

extern "C" {

const char* ap_status_string(ap_status s)
{
    switch (s) {
    case AP_OK: return "AP_OK";
    case AP_ERR_INVALID_ARG: return "AP_ERR_INVALID_ARG";
    case AP_ERR_UNSUPPORTED: return "AP_ERR_UNSUPPORTED";
    case AP_ERR_CAPACITY: return "AP_ERR_CAPACITY";
    case AP_ERR_HIP: return "AP_ERR_HIP";
    }
    return "AP_ERR_UNKNOWN";
}

int64_t ap_layout_max_tiles(int H, int Lq, int Lk, int block_m, int block_n)
{
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return -1;
    const int64_t nQB = (Lq + block_m - 1) / block_m, nKB = (Lk + block_n - 1) / block_n;
    return (int64_t)H * nQB * nKB;
}

size_t ap_layout_workspace_bytes(int H, int Lq, int Lk, int block_m, int block_n)
{
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return 0;
    size_t f, c, d, total;
    ap::layout_workspace_plan(H, Lq, Lk, block_m, block_n, &f, &c, &d, &total);
    return total;
}

static ap_status build_layout_common(const uint8_t* mask, long long stride_h, long long stride_row, int H,
                                     int Lq, int Lk, int block_m, int block_n, int32_t* row_ptr,
                                     int32_t* col_idx, uint64_t* bitmaps, int64_t cap, int64_t* nnz_out,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (H <= 0 || Lq <= 0 || Lk <= 0 || block_m <= 0 || block_n <= 0) return AP_ERR_INVALID_ARG;
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return AP_ERR_UNSUPPORTED;
    if (!mask || !row_ptr || !workspace) return AP_ERR_INVALID_ARG;
    if ((col_idx == nullptr) != (bitmaps == nullptr)) return AP_ERR_INVALID_ARG;
    if (col_idx && cap < 0) return AP_ERR_INVALID_ARG;
    if (!aligned(row_ptr, 4) || !aligned(col_idx, 4) || !aligned(bitmaps, 8) ||
        !aligned(nnz_out, 8) || !aligned(workspace, 8))
        return AP_ERR_INVALID_ARG;
    if (workspace_bytes < ap_layout_workspace_bytes(H, Lq, Lk, block_m, block_n)) return AP_ERR_CAPACITY;

    const hipError_t e = ap::launch_build_layout(mask, stride_h, stride_row, H, Lq, Lk, block_m, block_n,
                                                 row_ptr, col_idx, bitmaps, (long long)cap, nnz_out,
                                                 workspace, (hipStream_t)stream);
    return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

ap_status ap_build_layout(const uint8_t* mask, int H, int Lq, int Lk, int block_m, int block_n,
                          int32_t* row_ptr, int32_t* col_idx, uint64_t* bitmaps, int64_t cap,
                          int64_t* nnz_out, void* workspace, size_t workspace_bytes, void* stream)
{
    return build_layout_common(mask, (long long)Lq * Lk, Lk, H, Lq, Lk, block_m, block_n, row_ptr, col_idx,
                               bitmaps, cap, nnz_out, workspace, workspace_bytes, stream);
}

ap_status ap_build_layout_cropped(const uint8_t* mask, int H, int Lq_stored, int Lk_stored, int Lq, int Lk,
                                  int block_m, int block_n, int32_t* row_ptr, int32_t* col_idx,
                                  uint64_t* bitmaps, int64_t cap, int64_t* nnz_out, void* workspace,
                                  size_t workspace_bytes, void* stream)
{
    if (Lq_stored <= 0 || Lk_stored <= 0 || Lq > Lq_stored || Lk > Lk_stored) return AP_ERR_INVALID_ARG;
    return build_layout_common(mask, (long long)Lq_stored * Lk_stored, Lk_stored, H, Lq, Lk, block_m, block_n,
                               row_ptr, col_idx, bitmaps, cap, nnz_out, workspace, workspace_bytes, stream);
}

ap_status ap_build_layout_from_map(const float* abar, const float* tau, int H, int Lq, int Lk, int causal,
                                   int block_m, int block_n, int32_t* row_ptr, int32_t* col_idx,
                                   uint64_t* bitmaps, int64_t cap, int64_t* nnz_out, void* workspace,
                                   size_t workspace_bytes, void* stream)
{
    if (H <= 0 || Lq <= 0 || Lk <= 0 || block_m <= 0 || block_n <= 0) return AP_ERR_INVALID_ARG;
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return AP_ERR_UNSUPPORTED;
    if (block_n != 64) return AP_ERR_UNSUPPORTED;            // the attention kernels' window width
    if (!abar || !tau || !row_ptr || !workspace) return AP_ERR_INVALID_ARG;
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    if ((col_idx == nullptr) != (bitmaps == nullptr)) return AP_ERR_INVALID_ARG;
    if (col_idx && cap < 0) return AP_ERR_INVALID_ARG;
    if (!aligned(abar, 4) || !aligned(tau, 4) || !aligned(row_ptr, 4) || !aligned(col_idx, 4) ||
        !aligned(bitmaps, 8) || !aligned(nnz_out, 8) || !aligned(workspace, 8))
        return AP_ERR_INVALID_ARG;
    if (workspace_bytes < ap_layout_workspace_bytes(H, Lq, Lk, block_m, block_n)) return AP_ERR_CAPACITY;
    const hipError_t e = ap::launch_build_layout_from_map(abar, tau, causal ? 1 : 0, H, Lq, Lk, block_m, block_n,
                                                          row_ptr, col_idx, bitmaps, (long long)cap, nnz_out,
                                                          workspace, (hipStream_t)stream);
    return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

ap_status ap_build_schedule(const int32_t* row_ptr, const int32_t* col_idx, const uint64_t* bitmaps,
                            int H, int Lq, int Lk, int block_m, int block_n, int64_t cap, int causal,
                            int min_cols, const ap_schedule* sched, void* stream)
{
    if (!row_ptr || !col_idx || !bitmaps || !sched) return AP_ERR_INVALID_ARG;
    if (!sched->cnt || !sched->start || !sched->cols || !sched->bitmaps) return AP_ERR_INVALID_ARG;
    if (H <= 0 || Lq <= 0 || Lk <= 0 || cap < 0) return AP_ERR_INVALID_ARG;
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    if (min_cols < 0 || min_cols > 65) return AP_ERR_INVALID_ARG;
    if (block_n != 64 || !(block_m == 64 || block_m == 128)) return AP_ERR_UNSUPPORTED;
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return AP_ERR_UNSUPPORTED;
    if (!aligned(row_ptr, 4) || !aligned(col_idx, 4) || !aligned(bitmaps, 8) || !aligned(sched->cnt, 4) ||
        !aligned(sched->start, 4) || !aligned(sched->cols, 4) || !aligned(sched->bitmaps, 8))
        return AP_ERR_INVALID_ARG;
    ap::Schedule s{sched->cnt, sched->start, sched->cols, sched->bitmaps};
    const hipError_t e = ap::launch_build_schedule(row_ptr, col_idx, bitmaps, H, Lq, Lk, block_m,
                                                   (long long)cap, causal ? 1 : 0, min_cols == 0 ? 48 : min_cols, s,
                                                   (hipStream_t)stream);
    return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

size_t ap_fwd_split_workspace_bytes(int B, int H, int Lq, int D, int splits)
{
    if (B <= 0 || H <= 0 || Lq <= 0 || D <= 0 || splits <= 0) return 0;
    return (size_t)splits * (size_t)B * (size_t)H * (size_t)Lq * ((size_t)D + 1) * sizeof(float);
}

// splits = 0: the ordinary forward call; splits >= 1: the split variant with its workspace
static ap_status fwd_common(const void* Q, const void* K, const void* V, void* O, float* lse,
                            ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                            const int64_t* stride_q, const int64_t* stride_k,
                            const int64_t* stride_v, const int64_t* stride_o,
                            const int32_t* row_ptr, const int32_t* col_idx,
                            const uint64_t* bitmaps, int block_m, int block_n,
                            const ap_schedule* sched, int causal, float softmax_scale, int splits,
                            void* workspace, size_t workspace_bytes, void* stream, bool entmax = false,
                            bool decode = false, int Lq_layout = 0, int Lk_layout = 0)
{
    // cropped call: the layout (and schedule) were built for Lq_layout x Lk_layout, this call uses
    // the top-left Lq x Lk corner of that mask
    const bool cropped = Lq_layout > 0 || Lk_layout > 0;
    if (cropped) {
        if (Lq_layout < Lq || Lk_layout < Lk) return AP_ERR_INVALID_ARG;
        if (causal && Lk_layout < Lq_layout) return AP_ERR_INVALID_ARG;
        // a schedule has the causal limit of its own sizes folded into its bitmaps
        if (causal && sched && (long long)Lk - Lq != (long long)Lk_layout - Lq_layout) return AP_ERR_INVALID_ARG;
        if (dtype != AP_BF16) return AP_ERR_UNSUPPORTED;
    }
    if (!Q || !K || !V || !O || !stride_q || !stride_k || !stride_v || !stride_o || !row_ptr ||
        !col_idx || !bitmaps)
        return AP_ERR_INVALID_ARG;
    if (B <= 0 || H <= 0 || Lq <= 0 || Lk <= 0 || D <= 0 || block_m <= 0 || block_n <= 0)
        return AP_ERR_INVALID_ARG;
    if (dtype != AP_F32 && dtype != AP_BF16) return AP_ERR_INVALID_ARG;
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    if (O == Q || O == K || O == V) return AP_ERR_INVALID_ARG;
    if (isnan(softmax_scale) || isinf(softmax_scale)) return AP_ERR_INVALID_ARG;

    if (sched) {
        if (!sched->cnt || !sched->start || !sched->cols || !sched->bitmaps) return AP_ERR_INVALID_ARG;
        if (!aligned(sched->cnt, 4) || !aligned(sched->start, 4) || !aligned(sched->cols, 4) ||
            !aligned(sched->bitmaps, 8))
            return AP_ERR_INVALID_ARG;
        if (dtype != AP_BF16) return AP_ERR_UNSUPPORTED;
    }
    if (!(D == 32 || D == 64 || D == 128)) return AP_ERR_UNSUPPORTED;
    if (block_n != 64) return AP_ERR_UNSUPPORTED;
    if (!(block_m == 64 || (block_m == 128 && dtype == AP_BF16))) return AP_ERR_UNSUPPORTED;
    const long long nQB = (Lq + block_m - 1) / block_m;
    if (nQB * H * B >= 2147483647LL || H > 65535 || B > 65535) return AP_ERR_UNSUPPORTED;

    const int per16 = dtype == AP_BF16 ? 8 : 4;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) ||
        !aligned(lse, 4) || !aligned(row_ptr, 4) || !aligned(col_idx, 4) || !aligned(bitmaps, 8))
        return AP_ERR_INVALID_ARG;
    if (!strides_ok(stride_q, D, per16) || !strides_ok(stride_k, D, per16) ||
        !strides_ok(stride_v, D, per16) || !strides_ok(stride_o, D, per16))
        return AP_ERR_INVALID_ARG;

    // the matrix-core kernel addresses each (batch, head) slice of K and V with 32-bit byte offsets
    if (dtype == AP_BF16 && ((long long)Lk * stride_k[2] * 2 >= 2147483647LL ||
                             (long long)Lk * stride_v[2] * 2 >= 2147483647LL))
        return AP_ERR_UNSUPPORTED;

    // gathered rows are addressed as key * row stride with the 24-bit multiply
    if (sched && (Lk >= (1LL << 24) || stride_k[2] * 2 >= (1LL << 24) || stride_v[2] * 2 >= (1LL << 24)))
        return AP_ERR_UNSUPPORTED;

    if (entmax && (dtype != AP_BF16 || block_m != 64)) return AP_ERR_UNSUPPORTED;
    // one workgroup per query there
    if (decode && (dtype != AP_BF16 || sched || (long long)B * H * Lq >= 2147483647LL)) return AP_ERR_UNSUPPORTED;
    // bitmap rows are fetched with 32-bit byte offsets there: 512 bytes per tile
    if (entmax && nQB * ((Lk + 63) / 64) * H >= (1LL << 22)) return AP_ERR_UNSUPPORTED;
    if (splits > 0) {
        if (!workspace || !aligned(workspace, 16)) return AP_ERR_INVALID_ARG;
        if (dtype != AP_BF16 || (block_m != 64 && !decode)) return AP_ERR_UNSUPPORTED;
        if (splits > 1024 || nQB * H * B * splits >= 2147483647LL) return AP_ERR_UNSUPPORTED;
        if (decode && (long long)B * H * Lq * splits >= 2147483647LL) return AP_ERR_UNSUPPORTED;
        if (workspace_bytes < ap_fwd_split_workspace_bytes(B, H, Lq, D, splits)) return AP_ERR_CAPACITY;
    }

    ap::FwdArgs a;
    a.Q = Q; a.K = K; a.V = V; a.O = O; a.lse = lse;
    a.B = B; a.H = H; a.Lq = Lq; a.Lk = Lk; a.D = D;
    for (int k = 0; k < 3; ++k) {
        a.sq[k] = stride_q[k]; a.sk[k] = stride_k[k]; a.sv[k] = stride_v[k]; a.so[k] = stride_o[k];
    }
    a.row_ptr = row_ptr; a.col_idx = col_idx; a.bitmaps = bitmaps;
    a.block_m = block_m; a.block_n = block_n;
    a.causal = causal ? 1 : 0;
    a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
    if (sched)
        a.sched = ap::Schedule{sched->cnt, sched->start, sched->cols, sched->bitmaps};
    else
        a.sched = ap::Schedule{nullptr, nullptr, nullptr, nullptr};
    a.nqb_layout = (int)(((long long)(cropped ? Lq_layout : Lq) + block_m - 1) / block_m);
    a.crop = (cropped && Lk < Lk_layout) ? 1 : 0;
    a.splits = splits > 0 ? splits : 1;
    a.part_o = (float*)workspace;
    a.part_lse = a.part_o ? a.part_o + (size_t)a.splits * B * H * Lq * D : nullptr;

    hipError_t e;
    if (decode)
        e = ap::launch_fwd_decode(a, (hipStream_t)stream);
    else if (entmax)
        e = ap::launch_entmax15_fwd(a, lse, (hipStream_t)stream);
    else if (splits > 0)
        e = ap::launch_fwd_split(a, (hipStream_t)stream);
    else if (dtype == AP_BF16)
        e = ap::launch_fwd_mfma(a, (hipStream_t)stream);
    else
        e = ap::launch_fwd_valu(a, false, (hipStream_t)stream);
    return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

ap_status ap_sparse_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* lse,
                             ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                             const int64_t* stride_q, const int64_t* stride_k,
                             const int64_t* stride_v, const int64_t* stride_o,
                             const int32_t* row_ptr, const int32_t* col_idx,
                             const uint64_t* bitmaps, int block_m, int block_n,
                             const ap_schedule* sched, int causal, float softmax_scale, void* stream)
{
    return fwd_common(Q, K, V, O, lse, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v, stride_o,
                      row_ptr, col_idx, bitmaps, block_m, block_n, sched, causal, softmax_scale, 0,
                      nullptr, 0, stream);
}

ap_status ap_sparse_attn_fwd_cropped(const void* Q, const void* K, const void* V, void* O, float* lse,
                                     ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                     const int64_t* stride_q, const int64_t* stride_k,
                                     const int64_t* stride_v, const int64_t* stride_o,
                                     const int32_t* row_ptr, const int32_t* col_idx,
                                     const uint64_t* bitmaps, int block_m, int block_n, int Lq_layout,
                                     int Lk_layout, const ap_schedule* sched, int causal,
                                     float softmax_scale, void* stream)
{
    if (Lq_layout <= 0 || Lk_layout <= 0) return AP_ERR_INVALID_ARG;
    return fwd_common(Q, K, V, O, lse, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v, stride_o,
                      row_ptr, col_idx, bitmaps, block_m, block_n, sched, causal, softmax_scale, 0,
                      nullptr, 0, stream, false, false, Lq_layout, Lk_layout);
}

ap_status ap_sparse_attn_decode(const void* Q, const void* K, const void* V, void* O, float* lse,
                                ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                const int64_t* stride_q, const int64_t* stride_k,
                                const int64_t* stride_v, const int64_t* stride_o,
                                const int32_t* row_ptr, const int32_t* col_idx,
                                const uint64_t* bitmaps, int block_m, int block_n, int causal,
                                float softmax_scale, int splits, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    if (splits <= 0) return AP_ERR_INVALID_ARG;
    // one workgroup per query writes O itself: splits = 1 needs no workspace
    return fwd_common(Q, K, V, O, lse, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v, stride_o,
                      row_ptr, col_idx, bitmaps, block_m, block_n, nullptr, causal, softmax_scale,
                      splits > 1 ? splits : 0, splits > 1 ? workspace : nullptr, workspace_bytes, stream,
                      false, true);
}

ap_status ap_sparse_attn_entmax15_fwd(const void* Q, const void* K, const void* V, void* O, float* tau,
                                      ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                      const int64_t* stride_q, const int64_t* stride_k,
                                      const int64_t* stride_v, const int64_t* stride_o,
                                      const int32_t* row_ptr, const int32_t* col_idx,
                                      const uint64_t* bitmaps, int block_m, int block_n,
                                      const ap_schedule* sched, int causal, float softmax_scale,
                                      void* stream)
{
    return fwd_common(Q, K, V, O, tau, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v, stride_o,
                      row_ptr, col_idx, bitmaps, block_m, block_n, sched, causal, softmax_scale, 0,
                      nullptr, 0, stream, true);
}

ap_status ap_sparse_attn_fwd_split(const void* Q, const void* K, const void* V, void* O, float* lse,
                                   ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                   const int64_t* stride_q, const int64_t* stride_k,
                                   const int64_t* stride_v, const int64_t* stride_o,
                                   const int32_t* row_ptr, const int32_t* col_idx,
                                   const uint64_t* bitmaps, int block_m, int block_n,
                                   const ap_schedule* sched, int causal, float softmax_scale,
                                   int splits, void* workspace, size_t workspace_bytes, void* stream)
{
    if (splits <= 0) return AP_ERR_INVALID_ARG;
    return fwd_common(Q, K, V, O, lse, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v, stride_o,
                      row_ptr, col_idx, bitmaps, block_m, block_n, sched, causal, softmax_scale, splits,
                      workspace, workspace_bytes, stream);
}

ap_status ap_sparse_attn_fwd_split_static(const void* Q, const void* K, const void* V, void* O, float* lse,
                                          ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                          const int64_t* stride_q, const int64_t* stride_k,
                                          const int64_t* stride_v, const int64_t* stride_o,
                                          const int32_t* row_ptr, const int32_t* col_idx,
                                          const uint64_t* bitmaps, int block_m, int block_n,
                                          const ap_schedule* sched, int causal, float softmax_scale,
                                          int splits, void* stream)
{
    if (splits <= 0 || B <= 0 || H <= 0 || Lq <= 0 || D <= 0) return AP_ERR_INVALID_ARG;
    // the size check comes first and needs no GPU: 128-bit arithmetic cannot wrap for int arguments
    const unsigned __int128 need = (unsigned __int128)splits * (unsigned)B * (unsigned)H * (unsigned)Lq *
                                   ((unsigned)D + 1u) * sizeof(float);
    if (need > (unsigned __int128)AP_FWD_SPLIT_STATIC_MAX_BYTES) return AP_ERR_CAPACITY;
    void* ws = static_scratch();
    if (!ws) return AP_ERR_HIP;
    return fwd_common(Q, K, V, O, lse, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v, stride_o,
                      row_ptr, col_idx, bitmaps, block_m, block_n, sched, causal, softmax_scale, splits,
                      ws, AP_FWD_SPLIT_STATIC_MAX_BYTES, stream);
}

ap_status ap_build_layout_transpose(const int32_t* row_ptr, const int32_t* col_idx, int H, int Lq,
                                    int Lk, int block_m, int block_n, int64_t cap, int32_t* col_ptr,
                                    int32_t* row_idx, int32_t* tile_idx, void* stream)
{
    if (!row_ptr || !col_idx || !col_ptr || !row_idx || !tile_idx) return AP_ERR_INVALID_ARG;
    if (H <= 0 || Lq <= 0 || Lk <= 0 || cap < 0) return AP_ERR_INVALID_ARG;
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return AP_ERR_UNSUPPORTED;
    if (!aligned(row_ptr, 4) || !aligned(col_idx, 4) || !aligned(col_ptr, 4) || !aligned(row_idx, 4) ||
        !aligned(tile_idx, 4))
        return AP_ERR_INVALID_ARG;
    const int nQB = (Lq + block_m - 1) / block_m, nKB = (Lk + block_n - 1) / block_n;
    return ap::launch_layout_transpose(row_ptr, col_idx, H, nQB, nKB, cap, col_ptr, row_idx, tile_idx,
                                       (hipStream_t)stream) == hipSuccess ? AP_OK : AP_ERR_HIP;
}

size_t ap_bwd_workspace_bytes(int B, int H, int Lq)
{
    if (B <= 0 || H <= 0 || Lq <= 0) return 0;
    return (size_t)B * (size_t)H * (size_t)Lq * sizeof(float);
}

static ap_status bwd_common(const void* Q, const void* K, const void* V, const void* O,
                             const void* dO, const float* lse, void* dQ, void* dK, void* dV,
                             ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                             const int64_t* stride_q, const int64_t* stride_k,
                             const int64_t* stride_v, const int64_t* stride_o,
                             const int32_t* row_ptr, const int32_t* col_idx,
                             const uint64_t* bitmaps, const int32_t* col_ptr,
                             const int32_t* row_idx, const int32_t* tile_idx, int block_m,
                             int block_n, const ap_schedule* sched, const ap_schedule* col_sched, int causal,
                             float softmax_scale, void* workspace, size_t workspace_bytes, void* stream,
                             bool entmax = false)
{
    // 1.5-entmax: `lse` carries tau, there is no O (its role is taken by a pass over the entries),
    // and both schedules are required
    if (entmax) {
        if (O || !sched || !col_sched) return AP_ERR_INVALID_ARG;
        O = dO;                                              // keeps the shared checks below simple
    }
    if (!Q || !K || !V || !O || !dO || !lse || !dQ || !dK || !dV || !stride_q || !stride_k ||
        !stride_v || !stride_o || !row_ptr || !col_idx || !bitmaps || !col_ptr || !row_idx ||
        !tile_idx || !workspace)
        return AP_ERR_INVALID_ARG;
    if (B <= 0 || H <= 0 || Lq <= 0 || Lk <= 0 || D <= 0 || block_m <= 0 || block_n <= 0)
        return AP_ERR_INVALID_ARG;
    if (dtype != AP_F32 && dtype != AP_BF16) return AP_ERR_INVALID_ARG;
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    if (isnan(softmax_scale) || isinf(softmax_scale)) return AP_ERR_INVALID_ARG;
    const void* ins[5] = {Q, K, V, O, dO};
    for (const void* in : ins)
        if (dQ == in || dK == in || dV == in) return AP_ERR_INVALID_ARG;
    if (dQ == dK || dQ == dV || dK == dV) return AP_ERR_INVALID_ARG;
    if (dtype != AP_BF16) return AP_ERR_UNSUPPORTED;
    if (!(D == 32 || D == 64 || D == 128)) return AP_ERR_UNSUPPORTED;
    if (block_m != 64 || block_n != 64) return AP_ERR_UNSUPPORTED;
    const long long nQB = (Lq + 63) / 64, nKB = (Lk + 63) / 64;
    if (nQB * H * B >= 2147483647LL || nKB * H * B >= 2147483647LL) return AP_ERR_UNSUPPORTED;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(dO, 16) ||
        !aligned(dQ, 16) || !aligned(dK, 16) || !aligned(dV, 16) || !aligned(lse, 4) ||
        !aligned(row_ptr, 4) || !aligned(col_idx, 4) || !aligned(bitmaps, 8) || !aligned(col_ptr, 4) ||
        !aligned(row_idx, 4) || !aligned(tile_idx, 4) || !aligned(workspace, 16))
        return AP_ERR_INVALID_ARG;
    if (!strides_ok(stride_q, D, 8) || !strides_ok(stride_k, D, 8) || !strides_ok(stride_v, D, 8) ||
        !strides_ok(stride_o, D, 8))
        return AP_ERR_INVALID_ARG;
    // tiles of every operand are addressed with 32-bit byte offsets inside a (batch, head) slice
    if ((long long)Lk * stride_k[2] * 2 >= 2147483647LL || (long long)Lk * stride_v[2] * 2 >= 2147483647LL ||
        (long long)Lq * stride_q[2] * 2 >= 2147483647LL || (long long)Lq * stride_o[2] * 2 >= 2147483647LL)
        return AP_ERR_UNSUPPORTED;
    // bitmap rows are fetched with 32-bit byte offsets: 512 bytes per tile
    if (nQB * nKB * H >= (1LL << 22)) return AP_ERR_UNSUPPORTED;
    if (workspace_bytes < ap_bwd_workspace_bytes(B, H, Lq)) return AP_ERR_CAPACITY;
    // gathered rows (keys for one schedule, queries for the other) are addressed as row index * row
    // stride with the 24-bit multiply
    if ((sched || col_sched) &&
        (Lk >= (1LL << 24) || Lq >= (1LL << 24) || stride_k[2] * 2 >= (1LL << 24) || stride_v[2] * 2 >= (1LL << 24) ||
         stride_q[2] * 2 >= (1LL << 24) || stride_o[2] * 2 >= (1LL << 24)))
        return AP_ERR_UNSUPPORTED;
    for (const ap_schedule* sc : {sched, col_sched}) {
        if (!sc) continue;
        if (!sc->cnt || !sc->start || !sc->cols || !sc->bitmaps) return AP_ERR_INVALID_ARG;
        if (!aligned(sc->cnt, 4) || !aligned(sc->start, 4) || !aligned(sc->cols, 4) || !aligned(sc->bitmaps, 8))
            return AP_ERR_INVALID_ARG;
    }

    ap::BwdArgs a;
    a.Q = Q; a.K = K; a.V = V; a.O = O; a.dO = dO; a.lse = lse;
    a.dQ = dQ; a.dK = dK; a.dV = dV;
    a.B = B; a.H = H; a.Lq = Lq; a.Lk = Lk; a.D = D;
    for (int k = 0; k < 3; ++k) {
        a.sq[k] = stride_q[k]; a.sk[k] = stride_k[k]; a.sv[k] = stride_v[k]; a.so[k] = stride_o[k];
    }
    a.row_ptr = row_ptr; a.col_idx = col_idx; a.bitmaps = bitmaps;
    a.col_ptr = col_ptr; a.row_idx = row_idx; a.tile_idx = tile_idx;
    a.causal = causal ? 1 : 0;
    a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
    a.delta = (float*)workspace;
    a.sched = sched ? ap::Schedule{sched->cnt, sched->start, sched->cols, sched->bitmaps}
                    : ap::Schedule{nullptr, nullptr, nullptr, nullptr};
    a.csched = col_sched ? ap::Schedule{col_sched->cnt, col_sched->start, col_sched->cols, col_sched->bitmaps}
                         : ap::Schedule{nullptr, nullptr, nullptr, nullptr};
    a.entmax = entmax ? 1 : 0;
    if (entmax) {
        a.O = nullptr;
        return ap::launch_bwd_sched(a, true, true, (hipStream_t)stream) == hipSuccess ? AP_OK : AP_ERR_HIP;
    }
    return ap::launch_bwd(a, (hipStream_t)stream) == hipSuccess ? AP_OK : AP_ERR_HIP;
}

ap_status ap_sparse_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                             const void* dO, const float* lse, void* dQ, void* dK, void* dV,
                             ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                             const int64_t* stride_q, const int64_t* stride_k,
                             const int64_t* stride_v, const int64_t* stride_o,
                             const int32_t* row_ptr, const int32_t* col_idx,
                             const uint64_t* bitmaps, const int32_t* col_ptr,
                             const int32_t* row_idx, const int32_t* tile_idx, int block_m,
                             int block_n, int causal, float softmax_scale, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    return bwd_common(Q, K, V, O, dO, lse, dQ, dK, dV, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v,
                      stride_o, row_ptr, col_idx, bitmaps, col_ptr, row_idx, tile_idx, block_m, block_n,
                      nullptr, nullptr, causal, softmax_scale, workspace, workspace_bytes, stream);
}

ap_status ap_sparse_attn_bwd_sched(const void* Q, const void* K, const void* V, const void* O,
                                   const void* dO, const float* lse, void* dQ, void* dK, void* dV,
                                   ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                   const int64_t* stride_q, const int64_t* stride_k,
                                   const int64_t* stride_v, const int64_t* stride_o,
                                   const int32_t* row_ptr, const int32_t* col_idx,
                                   const uint64_t* bitmaps, const int32_t* col_ptr,
                                   const int32_t* row_idx, const int32_t* tile_idx, int block_m,
                                   int block_n, const ap_schedule* sched,
                                   const ap_schedule* col_sched, int causal, float softmax_scale,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    return bwd_common(Q, K, V, O, dO, lse, dQ, dK, dV, dtype, B, H, Lq, Lk, D, stride_q, stride_k, stride_v,
                      stride_o, row_ptr, col_idx, bitmaps, col_ptr, row_idx, tile_idx, block_m, block_n,
                      sched, col_sched, causal, softmax_scale, workspace, workspace_bytes, stream);
}

size_t ap_entmax15_bwd_workspace_bytes(int B, int H, int Lq)
{
    if (B <= 0 || H <= 0 || Lq <= 0) return 0;
    return (size_t)B * (size_t)H * (size_t)Lq * sizeof(float);
}

ap_status ap_sparse_attn_entmax15_bwd(const void* Q, const void* K, const void* V, const void* dO,
                                      const float* tau, void* dQ, void* dK, void* dV, ap_dtype dtype,
                                      int B, int H, int Lq, int Lk, int D, const int64_t* stride_q,
                                      const int64_t* stride_k, const int64_t* stride_v,
                                      const int64_t* stride_o, const int32_t* row_ptr,
                                      const int32_t* col_idx, const uint64_t* bitmaps,
                                      const int32_t* col_ptr, const int32_t* row_idx,
                                      const int32_t* tile_idx, int block_m, int block_n,
                                      const ap_schedule* sched, const ap_schedule* col_sched, int causal,
                                      float softmax_scale, void* workspace, size_t workspace_bytes,
                                      void* stream)
{
    return bwd_common(Q, K, V, nullptr, dO, tau, dQ, dK, dV, dtype, B, H, Lq, Lk, D, stride_q, stride_k,
                      stride_v, stride_o, row_ptr, col_idx, bitmaps, col_ptr, row_idx, tile_idx, block_m,
                      block_n, sched, col_sched, causal, softmax_scale, workspace, workspace_bytes, stream,
                      true);
}

ap_status ap_build_col_schedule(const int32_t* col_ptr, const int32_t* row_idx, const int32_t* tile_idx,
                                const uint64_t* bitmaps, int H, int Lq, int Lk, int block_m,
                                int block_n, int64_t cap, int causal, int min_rows,
                                const ap_schedule* col_sched, void* stream)
{
    if (!col_ptr || !row_idx || !tile_idx || !bitmaps || !col_sched) return AP_ERR_INVALID_ARG;
    if (!col_sched->cnt || !col_sched->start || !col_sched->cols || !col_sched->bitmaps) return AP_ERR_INVALID_ARG;
    if (H <= 0 || Lq <= 0 || Lk <= 0 || cap < 0) return AP_ERR_INVALID_ARG;
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    if (min_rows < 0 || min_rows > 65) return AP_ERR_INVALID_ARG;
    if (block_m != 64 || block_n != 64) return AP_ERR_UNSUPPORTED;
    if (!ap::layout_shape_ok(H, Lq, Lk, block_m, block_n)) return AP_ERR_UNSUPPORTED;
    if (!aligned(col_ptr, 4) || !aligned(row_idx, 4) || !aligned(tile_idx, 4) || !aligned(bitmaps, 8) ||
        !aligned(col_sched->cnt, 4) || !aligned(col_sched->start, 4) || !aligned(col_sched->cols, 4) ||
        !aligned(col_sched->bitmaps, 8))
        return AP_ERR_INVALID_ARG;
    ap::Schedule s{col_sched->cnt, col_sched->start, col_sched->cols, col_sched->bitmaps};
    const hipError_t e = ap::launch_build_col_schedule(col_ptr, row_idx, tile_idx, bitmaps, H, Lq, Lk,
                                                       causal ? 1 : 0, min_rows == 0 ? 48 : min_rows, s,
                                                       (hipStream_t)stream);
    return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

size_t ap_attention_maps_workspace_bytes(int B, int H, int Lq)
{
    if (B <= 0 || H <= 0 || Lq <= 0) return 0;
    return (size_t)B * (size_t)H * (size_t)Lq * sizeof(float);
}

static ap_status maps_common(const void* Q, const void* K, const float* lse, ap_dtype dtype, int B, int H,
                             int Lq, int Lk, int D, const int64_t* stride_q, const int64_t* stride_k,
                             int causal, float softmax_scale, float weight, float* abar, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    if (!Q || !K || !stride_q || !stride_k || !abar || !workspace) return AP_ERR_INVALID_ARG;
    if (B <= 0 || H <= 0 || Lq <= 0 || Lk <= 0 || D <= 0) return AP_ERR_INVALID_ARG;
    if (dtype != AP_F32 && dtype != AP_BF16) return AP_ERR_INVALID_ARG;
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    if (isnan(softmax_scale) || isinf(softmax_scale) || isnan(weight) || isinf(weight))
        return AP_ERR_INVALID_ARG;
    if (dtype != AP_BF16) return AP_ERR_UNSUPPORTED;
    if (!(D == 32 || D == 64 || D == 128)) return AP_ERR_UNSUPPORTED;
    const long long nQB = (Lq + 63) / 64, nKB = (Lk + 63) / 64;
    if (nQB * H * B >= 2147483647LL || nQB * nKB * H >= 2147483647LL) return AP_ERR_UNSUPPORTED;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(abar, 16) || !aligned(workspace, 16) || !aligned(lse, 4))
        return AP_ERR_INVALID_ARG;
    if (!strides_ok(stride_q, D, 8) || !strides_ok(stride_k, D, 8)) return AP_ERR_INVALID_ARG;
    if ((long long)Lk * stride_k[2] * 2 >= 2147483647LL) return AP_ERR_UNSUPPORTED;
    if (workspace_bytes < ap_attention_maps_workspace_bytes(B, H, Lq)) return AP_ERR_CAPACITY;

    ap::MapArgs a;
    a.Q = Q; a.K = K;
    a.B = B; a.H = H; a.Lq = Lq; a.Lk = Lk; a.D = D;
    for (int k = 0; k < 3; ++k) { a.sq[k] = stride_q[k]; a.sk[k] = stride_k[k]; }
    a.causal = causal ? 1 : 0;
    a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
    a.weight = weight;
    a.abar = abar;
    a.lse2 = (float*)workspace;
    return ap::launch_attention_maps(a, lse, (hipStream_t)stream) == hipSuccess ? AP_OK : AP_ERR_HIP;
}

ap_status ap_accumulate_attention_maps(const void* Q, const void* K, ap_dtype dtype, int B, int H,
                                       int Lq, int Lk, int D, const int64_t* stride_q,
                                       const int64_t* stride_k, int causal, float softmax_scale,
                                       float weight, float* abar, void* workspace,
                                       size_t workspace_bytes, void* stream)
{
    return maps_common(Q, K, nullptr, dtype, B, H, Lq, Lk, D, stride_q, stride_k, causal, softmax_scale,
                       weight, abar, workspace, workspace_bytes, stream);
}

ap_status ap_accumulate_attention_maps_lse(const void* Q, const void* K, const float* lse, ap_dtype dtype,
                                           int B, int H, int Lq, int Lk, int D, const int64_t* stride_q,
                                           const int64_t* stride_k, int causal, float softmax_scale,
                                           float weight, float* abar, void* workspace,
                                           size_t workspace_bytes, void* stream)
{
    if (!lse) return AP_ERR_INVALID_ARG;
    return maps_common(Q, K, lse, dtype, B, H, Lq, Lk, D, stride_q, stride_k, causal, softmax_scale,
                       weight, abar, workspace, workspace_bytes, stream);
}

size_t ap_prune_mask_workspace_bytes(void) { return ap::prune_mask_workspace_bytes(); }

ap_status ap_prune_mask(const float* abar, int H, int Lq, int Lk, int causal, double prune_fraction,
                        uint8_t* mask, float* tau_out, void* workspace, size_t workspace_bytes,
                        void* stream)
{
    if (!abar || (!mask && !tau_out) || !workspace) return AP_ERR_INVALID_ARG;
    if (H <= 0 || Lq <= 0 || Lk <= 0) return AP_ERR_INVALID_ARG;
    if (!(prune_fraction >= 0.0 && prune_fraction <= 1.0)) return AP_ERR_INVALID_ARG;   // also NaN
    if (causal && Lk < Lq) return AP_ERR_INVALID_ARG;
    // positions inside a pair of rows are 32-bit
    if ((long long)H * Lq >= 2147483647LL || Lk > (1 << 30)) return AP_ERR_UNSUPPORTED;
    if (!aligned(abar, 16) || !aligned(mask, 4) || !aligned(tau_out, 4) || !aligned(workspace, 16))
        return AP_ERR_INVALID_ARG;
    if (workspace_bytes < ap::prune_mask_workspace_bytes()) return AP_ERR_CAPACITY;

    // participating entries: every row's visible prefix
    unsigned long long N;
    if (causal) {
        // row i sees min(Lk, i + Lk - Lq + 1) = i + (Lk - Lq) + 1 keys (Lk >= Lq)
        const unsigned long long per_head =
            (unsigned long long)Lq * (unsigned long long)(Lk - Lq) +
            (unsigned long long)Lq * ((unsigned long long)Lq + 1ull) / 2ull;
        N = per_head * (unsigned long long)H;
    } else {
        N = (unsigned long long)H * (unsigned long long)Lq * (unsigned long long)Lk;
    }
    const double want = floor(prune_fraction * (double)N);
    const bool none = want >= (double)N;
    const unsigned long long rank = none ? 0ull : (unsigned long long)want;
    return ap::launch_prune_mask(abar, H, Lq, Lk, causal ? 1 : 0, rank, N, none, mask, tau_out, workspace,
                                 (hipStream_t)stream) == hipSuccess ? AP_OK : AP_ERR_HIP;
}

}  // extern "C"
