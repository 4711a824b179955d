// Backward pass of masked attention (gradients of the masked-attention equation of Section 3.2,
// needed by step 4 of its algorithm: training the pruned model).
//
//   P_ij  = exp(s_ij - lse_i) on kept, visible entries, 0 elsewhere
//   dV_j  = sum_i P_ij dO_i          dP_ij = <dO_i, V_j>          delta_i = <dO_i, O_i>
//   dS_ij = P_ij (dP_ij - delta_i)   dQ_i = scale sum_j dS_ij K_j  dK_j = scale sum_i dS_ij Q_i
//
// Three kernels, no floating-point atomics:
//   bwd_delta_kernel   delta_i for every (example, head, query)
//   bwd_dq_kernel      one workgroup per (example, head, block row): walks the row's tiles as the
//                      forward kernel does (a wavefront owns 32 queries, S^T = K Q^T and
//                      dP^T = V dO^T on the matrix cores, lane = query), dQ^T += K^T dS^T
//   bwd_dkv_kernel     one workgroup per (example, head, block column): walks the column's tiles
//                      through the transposed layout with the roles swapped (a wavefront owns 32
//                      keys, S = Q K^T and dP = dO V^T, lane = key), dV^T += dO^T P, dK^T += Q^T dS
// Both tile kernels recompute the scores from Q, K and the stored log-sum-exp; the products use
// the operand layouts, LDS swizzles and LDS-direct tile loads of the forward kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"
#include "ap_mfma_common.h"

namespace ap {

namespace {

using namespace mfma;

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// delta[b,h,i] = sum_d dO[b,h,i,d] * O[b,h,i,d]; one query per group of D/8 lanes.
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(BwdArgs a)
{
    constexpr int LPR = D / 8;                               // lanes per row, 8 elements each
    const long long rows = (long long)a.B * a.H * a.Lq;
    const long long row = ((long long)blockIdx.x * 256 + threadIdx.x) / LPR;
    const int part = threadIdx.x % LPR;
    float s = 0.f;
    if (row < rows) {
        const int i = (int)(row % a.Lq);
        const long long bh = row / a.Lq;
        const int h = (int)(bh % a.H);
        const long long b = bh / a.H;
        const size_t off = (size_t)b * a.so[0] + (size_t)h * a.so[1] + (size_t)i * a.so[2] + part * 8;
        const uint4 o = *reinterpret_cast<const uint4*>((const uint16_t*)a.O + off);
        const uint4 g = *reinterpret_cast<const uint4*>((const uint16_t*)a.dO + off);
        const uint32_t ow[4] = {o.x, o.y, o.z, o.w}, gw[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            s = fmaf(bf16_to_f32((uint16_t)ow[k]), bf16_to_f32((uint16_t)gw[k]), s);
            s = fmaf(bf16_to_f32((uint16_t)(ow[k] >> 16)), bf16_to_f32((uint16_t)(gw[k] >> 16)), s);
        }
    }
#pragma unroll
    for (int o = 1; o < LPR; o <<= 1) s += __shfl_xor(s, o, 64);
    if (row < rows && part == 0) a.delta[row] = s;
}

// log-sum-exp in base 2; a row without kept keys (lse = -inf) gets +inf, so that exp2(s - lse2) = 0
__device__ __forceinline__ float lse2_of(float lse) { return lse == -INFINITY ? INFINITY : lse * kLog2e; }

template <int D>
__global__ __launch_bounds__(128, 2) void bwd_dq_kernel(BwdArgs a, int nQB)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    __shared__ __attribute__((aligned(1024))) uint16_t smem[3 * TILE];
    lds_u16* Kk = (lds_u16*)smem;                            // K tile, key swizzle (rows x Q^T)
    lds_u16* Kv = Kk + TILE;                                 // K tile, value swizzle (K^T x dS^T)
    lds_u16* Vk = Kv + TILE;                                 // V tile, key swizzle (rows x dO^T)

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;

    const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int qb = nQB - 1 - (bid % nQB);
    const int h = (bid / nQB) % a.H;
    const int b = bid / (nQB * a.H);

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Gp = (const uint16_t*)a.dO + (size_t)b * a.so[0] + (size_t)h * a.so[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* dQp = (uint16_t*)a.dQ + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const int sk_bytes = (int)a.sk[2] * 2, sv_bytes = (int)a.sv[2] * 2;
    const rsrc_t k_rsrc = make_rsrc(Kp, (unsigned)((a.Lk - 1) * sk_bytes + D * 2));
    const rsrc_t v_rsrc = make_rsrc(Vp, (unsigned)((a.Lk - 1) * sv_bytes + D * 2));

    const int brow = wave * 32 + n;
    const int qrow = qb * 64 + brow;
    const bool row_ok = qrow < a.Lq;
    const int qload = row_ok ? qrow : a.Lq - 1;
    bf16x8 qreg[KSTEPS], greg[KSTEPS];                       // Q^T and dO^T operands
    {
        const uint16_t* qr = Qp + (size_t)qload * a.sq[2] + 8 * hh;
        const uint16_t* gr = Gp + (size_t)qload * a.so[2] + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            qreg[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
            greg[kk] = *reinterpret_cast<const bf16x8*>(gr + 16 * kk);
        }
    }
    const size_t stat = ((size_t)b * a.H + h) * a.Lq + qload;
    const float lse2 = row_ok ? lse2_of(a.lse[stat]) : INFINITY;
    const float delta = row_ok ? a.delta[stat] : 0.f;
    const float sc = a.scale * kLog2e;
    const long long diag = (long long)qrow + ((long long)a.Lk - a.Lq);
    const int k_swz = hh ^ swz_k<D>(n);
    const TrRead tr = make_tr_read<D>(lane);

    f32x16 dqacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;

    const int r = h * nQB + qb;
    const int t0 = a.row_ptr[r], t1 = a.row_ptr[r + 1];
    const long long block_diag = (long long)qb * 64 + 63 + ((long long)a.Lk - a.Lq);
    for (int t = t0; t < t1; ++t) {
        const int k0 = a.col_idx[t] * kBN;
        if (a.causal && k0 > block_diag) break;              // columns ascend: the rest is hidden too
        __syncthreads();                                     // the previous tile is consumed
        issue_tile_loads<D, 2, false>(k_rsrc, Kk, k0, sk_bytes, wave, lane);
        issue_tile_loads<D, 2, true>(k_rsrc, Kv, k0, sk_bytes, wave, lane);
        issue_tile_loads<D, 2, false>(v_rsrc, Vk, k0, sv_bytes, wave, lane);
        uint64_t word = a.bitmaps[(size_t)t * 64 + brow];
        wait_vmem();
        __syncthreads();
        if (a.causal) {
            const long long lim = diag - k0;
            if (lim < 0) word = 0;
            else if (lim < 63) word &= (2ull << lim) - 1ull;
        }
        f32x16 sacc[2], pacc[2];
        qk_64<D>(smem, qreg, n, k_swz, sacc);                // S^T  = K Q^T
        qk_64<D>(smem + 2 * TILE, greg, n, k_swz, pacc);     // dP^T = V dO^T
        const uint64_t wsh = word >> (4 * hh);
        const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int pos = 8 * (i / 4) + (i % 4);
                const float p = ((wbits[kb] >> pos) & 1u) ? __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], sc, -lse2)) : 0.f;
                sacc[kb][i] = p * (pacc[kb][i] - delta);     // dS^T
            }
        tr_mm_64<D>(Kv, sacc, dqacc, tr);                    // dQ^T += K^T dS^T
    }
    __syncthreads();                                         // all wavefronts are done with the tiles
    store_rows_bf16<D>(smem + wave * 32 * D, dqacc, a.scale, lane,
                       dQp + (size_t)(qb * 64 + wave * 32) * a.sq[2], a.sq[2], a.Lq - (qb * 64 + wave * 32));
}

template <int D>
__global__ __launch_bounds__(128, 1) void bwd_dkv_kernel(BwdArgs a, int nQB, int nKB)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    __shared__ __attribute__((aligned(1024))) uint16_t smem[4 * TILE];
    __shared__ __attribute__((aligned(16))) float s_lse2[64];
    __shared__ __attribute__((aligned(16))) float s_delta[64];
    __shared__ __attribute__((aligned(16))) uint64_t s_word[64];
    lds_u16* Qk = (lds_u16*)smem;                            // Q tile, key swizzle   (rows x K^T)
    lds_u16* Qv = Qk + TILE;                                 // Q tile, value swizzle (Q^T x dS)
    lds_u16* Gk = Qv + TILE;                                 // dO tile, key swizzle  (rows x V^T)
    lds_u16* Gv = Gk + TILE;                                 // dO tile, value swizzle (dO^T x P)

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;

    const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int kb = bid % nKB;
    const int h = (bid / nKB) % a.H;
    const int b = bid / (nKB * a.H);

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Gp = (const uint16_t*)a.dO + (size_t)b * a.so[0] + (size_t)h * a.so[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* dKp = (uint16_t*)a.dK + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    uint16_t* dVp = (uint16_t*)a.dV + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    const int sq_bytes = (int)a.sq[2] * 2, so_bytes = (int)a.so[2] * 2;
    const rsrc_t q_rsrc = make_rsrc(Qp, (unsigned)((a.Lq - 1) * sq_bytes + D * 2));
    const rsrc_t g_rsrc = make_rsrc(Gp, (unsigned)((a.Lq - 1) * so_bytes + D * 2));

    const int key = kb * 64 + wave * 32 + n;
    const int kload = key < a.Lk ? key : a.Lk - 1;
    bf16x8 kreg[KSTEPS], vreg[KSTEPS];                       // K^T and V^T operands
    {
        const uint16_t* kr = Kp + (size_t)kload * a.sk[2] + 8 * hh;
        const uint16_t* vr = Vp + (size_t)kload * a.sv[2] + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            kreg[kk] = *reinterpret_cast<const bf16x8*>(kr + 16 * kk);
            vreg[kk] = *reinterpret_cast<const bf16x8*>(vr + 16 * kk);
        }
    }
    const float sc = a.scale * kLog2e;
    const long long off = (long long)a.Lk - a.Lq;
    const int k_swz = hh ^ swz_k<D>(n);
    const TrRead tr = make_tr_read<D>(lane);
    const int kcol = wave * 32 + n;                          // this lane's key inside the tile

    f32x16 dkacc[DBLK], dvacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            dkacc[db][i] = 0.f;
            dvacc[db][i] = 0.f;
        }

    const int c = h * nKB + kb;
    const int c0 = a.col_ptr[c], c1 = a.col_ptr[c + 1];
    const size_t stat_base = ((size_t)b * a.H + h) * a.Lq;
    for (int ci = c0; ci < c1; ++ci) {
        const int qb = a.row_idx[ci];
        const int t = a.tile_idx[ci];
        const int q0 = qb * 64;
        if (a.causal && (long long)kb * 64 > (long long)q0 + 63 + off) continue;   // hidden from every row of the tile
        __syncthreads();                                     // the previous tile is consumed
        issue_tile_loads<D, 2, false>(q_rsrc, Qk, q0, sq_bytes, wave, lane);
        issue_tile_loads<D, 2, true>(q_rsrc, Qv, q0, sq_bytes, wave, lane);
        issue_tile_loads<D, 2, false>(g_rsrc, Gk, q0, so_bytes, wave, lane);
        issue_tile_loads<D, 2, true>(g_rsrc, Gv, q0, so_bytes, wave, lane);
        if (tid < 64) {                                      // per-query statistics and bitmap rows
            const int q = q0 + tid;
            const bool ok = q < a.Lq;
            s_lse2[tid] = ok ? lse2_of(a.lse[stat_base + q]) : INFINITY;
            s_delta[tid] = ok ? a.delta[stat_base + q] : 0.f;
            s_word[tid] = a.bitmaps[(size_t)t * 64 + tid];
        }
        wait_vmem();
        __syncthreads();
        f32x16 sacc[2], pacc[2];
        qk_64<D>(smem, kreg, n, k_swz, sacc);                // S  = Q K^T   (rows: queries, lane: key)
        qk_64<D>(smem + 2 * TILE, vreg, n, k_swz, pacc);     // dP = dO V^T
        const bool diag_tile = a.causal && (long long)kb * 64 + 63 > (long long)q0 + off;
#pragma unroll
        for (int qblk = 0; qblk < 2; ++qblk)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int r0 = 32 * qblk + 8 * g + 4 * hh;   // 4 consecutive query rows
                const float4 l4 = *reinterpret_cast<const float4*>(&s_lse2[r0]);
                const float4 d4 = *reinterpret_cast<const float4*>(&s_delta[r0]);
                const float le[4] = {l4.x, l4.y, l4.z, l4.w}, de[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * g + e;
                    bool kept = (s_word[r0 + e] >> kcol) & 1ull;
                    if (diag_tile) kept = kept && (long long)kb * 64 + kcol <= (long long)q0 + r0 + e + off;
                    const float p = kept ? __builtin_amdgcn_exp2f(fmaf(sacc[qblk][i], sc, -le[e])) : 0.f;
                    sacc[qblk][i] = p;                       // P
                    pacc[qblk][i] = p * (pacc[qblk][i] - de[e]);   // dS
                }
            }
        tr_mm_64<D>(Gv, sacc, dvacc, tr);                    // dV^T += dO^T P
        tr_mm_64<D>(Qv, pacc, dkacc, tr);                    // dK^T += Q^T dS
    }
    __syncthreads();                                         // all wavefronts are done with the tiles
    const int krow0 = kb * 64 + wave * 32;
    uint16_t* stage = smem + wave * 32 * D;
    store_rows_bf16<D>(stage, dkacc, a.scale, lane, dKp + (size_t)krow0 * a.sk[2], a.sk[2], a.Lk - krow0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the staging area is reused
    store_rows_bf16<D>(stage, dvacc, 1.0f, lane, dVp + (size_t)krow0 * a.sv[2], a.sv[2], a.Lk - krow0);
}

template <int D>
hipError_t launch_d(const BwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + 63) / 64, nKB = (a.Lk + 63) / 64;
    const long long rows = (long long)a.B * a.H * a.Lq;
    const long long dthreads = rows * (D / 8);
    hipLaunchKernelGGL(bwd_delta_kernel<D>, dim3((unsigned)((dthreads + 255) / 256)), dim3(256), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_dq_kernel<D>, dim3((unsigned)(a.B * a.H * nQB)), dim3(128), 0, stream, a, nQB);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_dkv_kernel<D>, dim3((unsigned)(a.B * a.H * nKB)), dim3(128), 0, stream, a, nQB, nKB);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd(const BwdArgs& a, hipStream_t stream)
{
    switch (a.D) {
        case 32: return launch_d<32>(a, stream);
        case 64: return launch_d<64>(a, stream);
        case 128: return launch_d<128>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ap
