// Masked attention forward for a handful of queries against a long key sequence (the cached
// memory of Section 4.1 taken to its limit: one new position, or a few, attends to everything
// before it under the layer's fixed mask).  Same result as ap_sparse_attn_fwd.
//
// With one to a few queries per (example, head) there is nothing for the matrix cores to do: a
// 64-query tile would be empty but for a row or two.  The work is reading the kept keys' K and V
// rows, so it is laid out for that: `splits` workgroups of 16 wavefronts per query, each with a
// contiguous share of the stored tiles of the query's block row; the lanes of a wavefront span the
// head dimension (one K row or V row is one coalesced read of the wavefront); the wavefronts
// share out the workgroup's tiles, walk the set bits of the query's bitmap words, and each keeps
// an online softmax over its keys in fp32; the 16 partial results are merged through LDS, and
// those of several workgroups by the split forward call's merge kernel.  Keys are taken eight at
// a time, so that sixteen row reads are in flight per wavefront.
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

// Sum over the 64 lanes with data-parallel-primitive moves (register to register, no LDS
// round trip per step): pairs, quads, half rows and rows by mirrored exchanges, then the row
// totals are passed on to the following rows; lane 63 ends up with the total, which is returned
// to every lane.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_step(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
    return v + __int_as_float(moved);
}
__device__ __forceinline__ float wave_sum(float v)
{
    v = dpp_step<0xB1, 0xf>(v);                              // quad_perm [1,0,3,2]
    v = dpp_step<0x4E, 0xf>(v);                              // quad_perm [2,3,0,1]
    v = dpp_step<0x141, 0xf>(v);                             // row_half_mirror
    v = dpp_step<0x140, 0xf>(v);                             // row_mirror: every lane holds its row's sum
    v = dpp_step<0x142, 0xa>(v);                             // row_bcast15 into rows 1 and 3
    v = dpp_step<0x143, 0xc>(v);                             // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// A lane holds E = 2 consecutive elements of a row (D = 128), 1 (D = 64), or 1 on the first 32
// lanes (D = 32): LPR = D / E lanes carry a row.
template <int D>
__global__ __launch_bounds__(64 * kWaves) void decode_kernel(FwdArgs a, int nQB)
{
    constexpr int E = D == 128 ? 2 : 1;
    constexpr int LPR = D / E;
    constexpr int U = 8;                                     // keys per step
    __shared__ float s_m[kWaves], s_l[kWaves];
    __shared__ float s_o[kWaves][D];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x % a.splits;
    const int row_id = blockIdx.x / a.splits;
    const int i = row_id % a.Lq;                             // query
    const int h = (row_id / a.Lq) % a.H;
    const int b = row_id / (a.Lq * a.H);
    const bool live = lane < LPR;                            // lanes that carry row elements

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1] + (size_t)i * a.sq[2];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];

    // one row's elements of this lane, as fp32
    auto load_row = [&](const uint16_t* row, float* x) {
        if (E == 2) {
            const uint32_t w = live ? *reinterpret_cast<const uint32_t*>(row + 2 * lane) : 0u;
            x[0] = bf16_lo(w);
            x[E - 1] = bf16_hi(w);
        } else {
            x[0] = live ? bf16_lo(row[lane]) : 0.f;
        }
    };

    float q[E];
    load_row(Qp, q);
    const float sc = a.scale * kLog2e;
#pragma unroll
    for (int e = 0; e < E; ++e) q[e] *= sc;                  // scores come out in the log2 domain

    float m = -INFINITY, l = 0.f;                            // wave-uniform running maximum and sum
    float o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.f;

    const int r = h * nQB + i / a.block_m;
    const int rr = i % a.block_m;
    const long long diag = (long long)i + ((long long)a.Lk - a.Lq);
    int t0 = a.row_ptr[r], t1 = a.row_ptr[r + 1];
    {                                                        // this workgroup's share of the tiles
        const int per = (t1 - t0 + a.splits - 1) / a.splits;
        t0 = min(t1, t0 + split * per);
        t1 = min(t1, t0 + per);
    }

    auto fold = [&](const int* key, int n) {                 // n <= U keys, wave-uniform
        float kx[U][E], vx[U][E];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < n) {
                load_row(Kp + (size_t)key[u] * a.sk[2], kx[u]);
                load_row(Vp + (size_t)key[u] * a.sv[2], vx[u]);
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < n) {
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) part = fmaf(q[e], kx[u][e], part);
                const float s = wave_sum(part);
                const float m_new = fmaxf(m, s);
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);   // 0 when m was -inf
                const float p = __builtin_amdgcn_exp2f(s - m_new);
                l = fmaf(l, alpha, p);
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = fmaf(o[e], alpha, p * vx[u][e]);
                m = m_new;
            }
    };

    // The workgroup's tiles are dealt to the wavefronts in contiguous groups of G <= 64; a group's
    // block columns and bitmap words are fetched with one load per lane, so that the walk over the
    // kept keys does not wait for memory once per tile.
    int key[U], nkey = 0;
    const int G = min(64, max(1, (t1 - t0 + kWaves - 1) / kWaves));
    for (int base = t0 + wave * G; base < t1; base += kWaves * G) {
        const int t = base + lane;
        int k0_v = 0;
        uint64_t word_v = 0;
        if (lane < G && t < t1) {
            k0_v = a.col_idx[t] * 64;
            word_v = a.bitmaps[(size_t)t * a.block_m + rr];
            if (a.causal) {
                const long long lim = diag - k0_v;
                if (lim < 0) word_v = 0;
                else if (lim < 63) word_v &= (2ull << lim) - 1ull;
            }
        }
        unsigned long long tiles = __ballot(word_v != 0);
        while (tiles) {
            const int src = __ffsll((long long)tiles) - 1;
            tiles &= tiles - 1;
            const int k0 = __builtin_amdgcn_readlane(k0_v, src);
            uint64_t word = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(word_v >> 32), src) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)word_v, src);
            while (word) {
                const int j = __ffsll((long long)word) - 1;
                word &= word - 1;
#pragma unroll
                for (int u = 0; u < U; ++u)                  // key[nkey] = k0 + j without indexing registers
                    if (u == nkey) key[u] = k0 + j;
                if (++nkey == U) {
                    fold(key, U);
                    nkey = 0;
                }
            }
        }
    }
    if (nkey > 0) fold(key, nkey);

    // merge the wavefronts' partial results: O = sum_w 2^(m_w - M) o_w / sum_w 2^(m_w - M) l_w
    if (lane == 0) {
        s_m[wave] = m;
        s_l[wave] = l;
    }
    if (live) {
#pragma unroll
        for (int e = 0; e < E; ++e) s_o[wave][E * lane + e] = o[e];
    }
    __syncthreads();
    if (wave == 0) {
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
                for (int e = 0; e < E; ++e) acc[e] = fmaf(s_o[w][E * lane + e], f, acc[e]);
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
