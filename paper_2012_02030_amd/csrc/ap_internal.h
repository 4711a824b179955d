// Declarations shared by the library's own translation units (never by the test oracle).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ap {

// ---- layout pass (ap_layout.hip)
bool layout_shape_ok(int H, int Lq, int Lk, int BM, int BN);
void layout_workspace_plan(int H, int Lq, int Lk, int BM, int BN, size_t* flags_off,
                           size_t* counts_off, size_t* dense_off, size_t* total);
// mask[h, i, j] is the byte at h * stride_h + i * stride_row + j
hipError_t launch_build_layout(const uint8_t* mask, long long stride_h, long long stride_row, int H,
                               int Lq, int Lk, int BM, int BN, int32_t* row_ptr, int32_t* col_idx,
                               uint64_t* bitmaps, long long cap, int64_t* nnz_out, void* workspace,
                               hipStream_t stream);

// the same from the fp32 mean map and the layer's threshold (device scalar): kept iff not
// (abar < tau) and, if causal, j <= i + (Lk - Lq); 64-key windows only
hipError_t launch_build_layout_from_map(const float* abar, const float* tau, int causal, int H, int Lq, int Lk,
                                        int BM, int BN, int32_t* row_ptr, int32_t* col_idx, uint64_t* bitmaps,
                                        long long cap, int64_t* nnz_out, void* workspace, hipStream_t stream);

// ---- visit schedule (ap_schedule.hip): entry e of block row r is element row_ptr[r] + e
struct Schedule {
    int32_t* cnt;        // [H*nQB]      entries of each block row
    int32_t* start;      // [cap]        >= 0: first key of 64 consecutive keys; -1: gathered keys
    int32_t* cols;       // [cap*64]     key of every slot of a gathered entry (Lk = empty slot)
    uint64_t* bitmaps;   // [cap*BM]     bit c of row rr: slot c kept (causal limit folded in)
};
hipError_t launch_build_schedule(const int32_t* row_ptr, const int32_t* col_idx,
                                 const uint64_t* bitmaps, int H, int Lq, int Lk, int BM,
                                 long long cap, int causal, int min_cols, const Schedule& s,
                                 hipStream_t stream);

// ---- attention forward (ap_attn_valu.hip, ap_attn_mfma.hip)
struct FwdArgs {
    const void* Q;
    const void* K;
    const void* V;
    void* O;
    float* lse;                     // may be null
    int B, H, Lq, Lk, D;
    long long sq[3], sk[3], sv[3], so[3];   // element strides: batch, head, sequence
    const int32_t* row_ptr;
    const int32_t* col_idx;
    const uint64_t* bitmaps;
    int block_m, block_n;
    int causal;
    float scale;                    // already resolved (> 0)
    Schedule sched;                 // all null: walk the layout itself
    int nqb_layout;                 // block rows per head of the layout (> those of Lq for a cropped call)
    int crop;                       // 1: the layout covers more keys than Lk; keys >= Lk are hidden
    int splits;                     // split path only: chunks per block row
    float* part_o;                  // [splits, B, H, Lq, D] fp32 partial outputs
    float* part_lse;                // [splits, B, H, Lq]
};

// fp32-arithmetic kernel (one query per lane); handles fp32 and bf16 storage, block 64x64
hipError_t launch_fwd_valu(const FwdArgs& a, bool bf16, hipStream_t stream);
// bf16 matrix-core kernel; block_m 64 or 128, block_n 64
hipError_t launch_fwd_mfma(const FwdArgs& a, hipStream_t stream);
// same result, the entries of every block row cut into a.splits chunks and merged (block_m 64)
hipError_t launch_fwd_split(const FwdArgs& a, hipStream_t stream);

// merges the a.splits partial results in a.part_o / a.part_lse into O and lse (ap_attn_mfma.hip)
hipError_t launch_merge_splits(const FwdArgs& a, hipStream_t stream);
// a few queries against many keys, a.splits workgroups per query, no matrix cores (ap_attn_decode.hip)
hipError_t launch_fwd_decode(const FwdArgs& a, hipStream_t stream);

// ---- 1.5-entmax forward (ap_attn_entmax.hip): bf16, block 64x64, plain layout walk
hipError_t launch_entmax15_fwd(const FwdArgs& a, float* tau_out, hipStream_t stream);

// ---- backward pass (ap_layout_transpose.hip, ap_attn_bwd.hip)
hipError_t launch_layout_transpose(const int32_t* row_ptr, const int32_t* col_idx, int H, int nQB,
                                   int nKB, long long cap, int32_t* col_ptr, int32_t* row_idx,
                                   int32_t* tile_idx, hipStream_t stream);
struct BwdArgs {
    const void* Q;
    const void* K;
    const void* V;
    const void* O;
    const void* dO;
    const float* lse;
    void* dQ;
    void* dK;
    void* dV;
    int B, H, Lq, Lk, D;
    long long sq[3], sk[3], sv[3], so[3];   // element strides: batch, head, sequence
    const int32_t* row_ptr;
    const int32_t* col_idx;
    const uint64_t* bitmaps;
    const int32_t* col_ptr;
    const int32_t* row_idx;
    const int32_t* tile_idx;
    int causal;
    float scale;                    // already resolved (> 0)
    float* delta;                   // [B, H, Lq] scratch: sum_d dO * O of each row
    Schedule sched;                 // row schedule for dQ; all null: walk the layout
    Schedule csched;                // column schedule for dK, dV; all null: walk the transposed layout
    int entmax;                     // 1: 1.5-entmax (both schedules required; lse holds tau, delta gets gbar)
};
hipError_t launch_bwd(const BwdArgs& a, hipStream_t stream);
// the kernels that walk schedules (ap_attn_bwd_sched.hip); softmax: delta must have been computed;
// entmax: runs the gbar pass and both gradient kernels whatever dq and dkv say
hipError_t launch_bwd_sched(const BwdArgs& a, bool dq, bool dkv, hipStream_t stream);
// column schedule (ap_col_schedule.hip): entry e of block column c is element col_ptr[c] + e
hipError_t launch_build_col_schedule(const int32_t* col_ptr, const int32_t* row_idx, const int32_t* tile_idx,
                                     const uint64_t* bitmaps, int H, int Lq, int Lk, int causal,
                                     int min_rows, const Schedule& s, hipStream_t stream);

// ---- mask construction: mean attention map (ap_maps.hip)
struct MapArgs {
    const void* Q;
    const void* K;
    int B, H, Lq, Lk, D;
    long long sq[3], sk[3];         // element strides: batch, head, sequence
    int causal;
    float scale;                    // already resolved (> 0)
    float weight;
    float* abar;                    // [H, Lq, Lk], accumulated into
    float* lse2;                    // [B, H, Lq] scratch: base-2 log-sum-exp of each score row
};
// lse: null (the row statistics are computed by a pass of their own), or the natural-log
// log-sum-exp [B, H, Lq] of the same scores, as the attention forward call returns it
hipError_t launch_attention_maps(const MapArgs& a, const float* lse, hipStream_t stream);

// ---- mask construction: percentile threshold and mask (ap_threshold.hip)
size_t prune_mask_workspace_bytes();
// rank: 0-based position of tau among the n participating entries; none: prune everything
hipError_t launch_prune_mask(const float* abar, int H, int Lq, int Lk, int causal,
                             unsigned long long rank, unsigned long long n, bool none, uint8_t* mask,
                             float* tau_out, void* workspace, hipStream_t stream);

}  // namespace ap
