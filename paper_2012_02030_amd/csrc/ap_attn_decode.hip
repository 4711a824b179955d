// Masked attention forward for a handful of queries against a long key sequence (the cached
// memory of Section 4.1 taken to its limit: one new position, or a few, attends to everything
// before it under the layer's fixed mask).  Same result as ap_sparse_attn_fwd.
//
// With one to a few queries per (example, head) there is nothing for the matrix cores to do: a
// 64-query tile would be empty but for a row or two.  The work is reading the kept keys' K and V
// rows, so it is laid out for that.  `splits` workgroups of 16 wavefronts per query, each with a
// contiguous share of the stored tiles of the query's block row.  A workgroup
//   1. turns the bitmap words of up to 128 tiles at a time into the list of kept visible keys in
//      LDS (one thread per tile, a prefix sum of the population counts gives every thread its
//      place in the list), so that what follows is a flat loop over keys;
//   2. runs one online-softmax stream per group of D / 8 lanes: a lane holds 8 elements of the
//      query and of the output, a K or V row is one 16-byte load per lane of the group (a
//      wavefront instruction fetches 64 / (D / 8) rows), the dot product is 8 multiply-adds and a
//      sum over the group with data-parallel-primitive moves inside a 16-lane row; stream s takes
//      keys s, s + S, s + 2 S, ... of the list, four keys of every stream are in flight at a time;
//   3. merges the streams of a wavefront by lane exchanges, the 16 wavefronts through LDS, and
//      those of several workgroups by the split forward call's merge kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

constexpr int kWaves = 16;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(moved);
}
// Sum over aligned groups of LPK = 4, 8 or 16 lanes; every lane of a group gets the group's sum.
template <int LPK>
__device__ __forceinline__ float group_sum(float v)
{
    v = dpp_add<0xB1>(v);                                    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);                                    // quad_perm [2,3,0,1]
    if (LPK >= 8) v = dpp_add<0x141>(v);                     // row_half_mirror
    if (LPK >= 16) v = dpp_add<0x140>(v);                    // row_mirror
    return v;
}

// 2^(a - b) for a <= b, with 2^(-inf - -inf) = 1 (a stream that has seen no key keeps its zeros)
__device__ __forceinline__ float scale_to(float a, float b)
{
    return a == b ? 1.0f : __builtin_amdgcn_exp2f(a - b);
}

template <int D>
__global__ __launch_bounds__(64 * kWaves) void decode_kernel(FwdArgs a, int nQB)
{
    constexpr int LPK = D / 8;                               // lanes per key row
    constexpr int SPW = 64 / LPK;                            // streams per wavefront
    constexpr int NS = kWaves * SPW;                         // streams per workgroup
    constexpr int CHUNK = 128;                               // tiles per pass
    constexpr int LCAP = CHUNK * 64;                         // keys per pass at most
    constexpr int UN = 4;                                    // keys of a stream in flight
    constexpr int E = D == 128 ? 2 : 1;                      // final merge: elements per lane
    static_assert(kWaves * D <= LCAP, "the merge area reuses the key list");
    __shared__ int s_list[LCAP];                             // kept visible keys; later the merge area
    __shared__ int s_wsum[2];
    __shared__ float s_m[kWaves], s_l[kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane % LPK;                              // which 8 elements of a row
    const int strm = wave * SPW + lane / LPK;                // this lane's stream
    const int split = blockIdx.x % a.splits;
    const int row_id = blockIdx.x / a.splits;
    const int i = row_id % a.Lq;                             // query
    const int h = (row_id / a.Lq) % a.H;
    const int b = row_id / (a.Lq * a.H);

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1] + (size_t)i * a.sq[2];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];

    auto unpack8 = [](const uint4& w, float* x) {
        x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
        x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
    };

    float q[8];
    {
        const uint4 w = *reinterpret_cast<const uint4*>(Qp + 8 * sub);
        unpack8(w, q);
        const float sc = a.scale * kLog2e;                   // scores come out in the log2 domain
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] *= sc;
    }
    float m = -INFINITY, l = 0.f;                            // this stream's running maximum and sum
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;

    const int r = h * nQB + i / a.block_m;
    const int rr = i % a.block_m;
    const long long diag = (long long)i + ((long long)a.Lk - a.Lq);
    int t0 = a.row_ptr[r], t1 = a.row_ptr[r + 1];
    {                                                        // this workgroup's share of the tiles
        const int per = (t1 - t0 + a.splits - 1) / a.splits;
        t0 = min(t1, t0 + split * per);
        t1 = min(t1, t0 + per);
    }

    for (int c0 = t0; c0 < t1; c0 += CHUNK) {                // workgroup-uniform trip count
        // ---- 1. the kept visible keys of tiles c0 .. c0 + CHUNK - 1, ascending, into s_list
        uint64_t word = 0;
        int k0 = 0;
        if (tid < CHUNK && c0 + tid < t1) {
            const int t = c0 + tid;
            k0 = a.col_idx[t] * 64;
            word = a.bitmaps[(size_t)t * a.block_m + rr];
            if (a.causal) {
                const long long lim = diag - k0;
                if (lim < 0) word = 0;
                else if (lim < 63) word &= (2ull << lim) - 1ull;
            }
        }
        const int cnt = __popcll(word);
        int incl = cnt;                                      // inclusive prefix sum inside the wavefront
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (wave < 2 && lane == 63) s_wsum[wave] = incl;     // CHUNK = 128 tiles: two wavefronts hold them
        __syncthreads();                                     // also: the previous pass is done with s_list
        const int n = s_wsum[0] + s_wsum[1];                 // keys of this pass
        {
            int pos = incl - cnt + (wave == 1 ? s_wsum[0] : 0);
            while (word) {
                const int j = __ffsll((long long)word) - 1;
                word &= word - 1;
                s_list[pos++] = k0 + j;
            }
        }
        __syncthreads();

        // ---- 2. stream `strm` folds keys strm, strm + NS, ... of the list
        for (int base = 0; base < n; base += UN * NS) {
            uint4 kx[UN], vx[UN];
            bool valid[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int idx = base + u * NS + strm;
                valid[u] = idx < n;
                const int key = s_list[valid[u] ? idx : 0];  // n > 0 here: slot 0 is a real key
                kx[u] = *reinterpret_cast<const uint4*>(Kp + (size_t)key * a.sk[2] + 8 * sub);
                vx[u] = *reinterpret_cast<const uint4*>(Vp + (size_t)key * a.sv[2] + 8 * sub);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                float x[8];
                unpack8(kx[u], x);
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) part = fmaf(q[e], x[e], part);
                const float s = group_sum<LPK>(part);
                const float m_new = valid[u] ? fmaxf(m, s) : m;
                const float alpha = scale_to(m, m_new);
                const float p = valid[u] ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
                l = fmaf(l, alpha, p);
                unpack8(vx[u], x);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = fmaf(o[e], alpha, p * x[e]);
                m = m_new;
            }
        }
    }

    // ---- 3. merge: the streams of a wavefront by lane exchanges ...
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m, off, 64);
        const float l2 = __shfl_xor(l, off, 64);
        const float M = fmaxf(m, m2);
        const float f1 = scale_to(m, M), f2 = scale_to(m2, M);
        l = l * f1 + l2 * f2;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = o[e] * f1 + __shfl_xor(o[e], off, 64) * f2;
        m = M;
    }
    // ... the wavefronts through LDS: O = sum_w 2^(m_w - M) o_w / sum_w 2^(m_w - M) l_w
    __syncthreads();                                         // everybody is done with the key list
    float* s_o = reinterpret_cast<float*>(s_list);           // [kWaves][D]
    if (lane == 0) {
        s_m[wave] = m;
        s_l[wave] = l;
    }
    if (lane < LPK) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s_o[wave * D + 8 * lane + e] = o[e];
    }
    __syncthreads();
    if (wave == 0) {
        const bool live = lane < D / E;                      // lanes that carry row elements
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, s_m[w]);
        float L = 0.f, acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;
        for (int w = 0; w < kWaves; ++w) {
            const float f = s_m[w] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s_m[w] - M);
            L = fmaf(s_l[w], f, L);
            if (live) {
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] = fmaf(s_o[w * D + E * lane + e], f, acc[e]);
            }
        }
        const float inv = L > 0.f ? 1.f / L : 0.f;           // no visible kept key: O = 0
        const float lse = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -INFINITY;
        if (a.splits > 1) {                                  // normalised fp32 partial result for the merge
            const size_t prow = (((size_t)split * a.B + b) * a.H + h) * a.Lq + i;
            if (live) {
#pragma unroll
                for (int e = 0; e < E; ++e) a.part_o[prow * D + E * lane + e] = acc[e] * inv;
            }
            if (lane == 0) a.part_lse[prow] = lse;
            return;
        }
        uint16_t* Op = (uint16_t*)a.O + (size_t)b * a.so[0] + (size_t)h * a.so[1] + (size_t)i * a.so[2];
        if (live) {
            if (E == 2)
                *reinterpret_cast<uint32_t*>(Op + 2 * lane) = bf16_rne(acc[0] * inv) | (bf16_rne(acc[E - 1] * inv) << 16);
            else
                Op[lane] = (uint16_t)bf16_rne(acc[0] * inv);
        }
        if (a.lse && lane == 0) a.lse[((size_t)b * a.H + h) * a.Lq + i] = lse;
    }
}

}  // namespace

hipError_t launch_fwd_decode(const FwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + a.block_m - 1) / a.block_m;
    const dim3 grid((unsigned)((long long)a.B * a.H * a.Lq * a.splits)), block(64 * kWaves);
    switch (a.D) {
        case 32: hipLaunchKernelGGL(decode_kernel<32>, grid, block, 0, stream, a, nQB); break;
        case 64: hipLaunchKernelGGL(decode_kernel<64>, grid, block, 0, stream, a, nQB); break;
        case 128: hipLaunchKernelGGL(decode_kernel<128>, grid, block, 0, stream, a, nQB); break;
        default: return hipErrorInvalidValue;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1) return e;
    return launch_merge_splits(a, stream);
}

}  // namespace ap
