// Backward pass of masked attention (gradients of the masked-attention equation of Section 3.2,
// needed by step 4 of its algorithm: training the pruned model).
//
//   P_ij  = exp(s_ij - lse_i) on kept, visible entries, 0 elsewhere
//   dV_j  = sum_i P_ij dO_i          dP_ij = <dO_i, V_j>          delta_i = <dO_i, O_i>
//   dS_ij = P_ij (dP_ij - delta_i)   dQ_i = scale sum_j dS_ij K_j  dK_j = scale sum_i dS_ij Q_i
//
// Three kernels, no floating-point atomics:
//   bwd_delta_kernel   delta_i for every (example, head, query)
//   bwd_dq_kernel      one workgroup per (example, head, two block rows): walks the rows' tiles as
//                      the forward kernel does (a wavefront owns 32 queries, S^T = K Q^T and
//                      dP^T = V dO^T on the matrix cores, lane = query), dQ^T += K^T dS^T
//   bwd_dkv_kernel     one workgroup per (example, head, two block columns): walks the columns'
//                      tiles through the transposed layout with the roles swapped (a wavefront owns
//                      32 keys, S = Q K^T and dP = dO V^T, lane = key), dV^T += dO^T P, dK^T += Q^T dS
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

// Two ascending index lists walked together: at every step the smaller head (or both, if
// equal) is taken.  All values are wave-uniform.
struct Merge {
    int ia, a1, ib, b1;          // cursors and ends of the two lists
    int key;                     // current index value (block column or block row); INT_MAX: done
    int ta, tb;                  // positions in the lists of the current step, -1 if absent
};

__device__ __forceinline__ void merge_step(Merge& m, const int32_t* list)
{
    const int ca = m.ia < m.a1 ? list[m.ia] : 0x7fffffff;
    const int cb = m.ib < m.b1 ? list[m.ib] : 0x7fffffff;
    m.key = ca < cb ? ca : cb;
    m.ta = (ca == m.key && ca != 0x7fffffff) ? m.ia++ : -1;
    m.tb = (cb == m.key && cb != 0x7fffffff) ? m.ib++ : -1;
}

// dQ: one workgroup per (example, head, pair of block rows); wavefronts 0,1 own the 64 queries of
// the first block row, wavefronts 2,3 those of the second.  The tiles of both block rows are
// walked together in ascending column order, so a K/V tile that both need is loaded once.  Two
// LDS stages: the next tile travels while the current one is computed, one barrier per tile.
template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dq_kernel(BwdArgs a, int nQB, int nQP)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    constexpr int STAGE = 3 * TILE + 512;                    // Kk, Kv, Vk, bitmap words of both block rows
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * STAGE];
    lds_u16* lds = (lds_u16*)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;
    const int half = wave >> 1;                              // which block row of the pair

    const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int qp = nQP - 1 - (bid % nQP);                    // long causal rows first
    const int h = (bid / nQP) % a.H;
    const int b = bid / (nQP * a.H);
    const int qb = 2 * qp + half;
    const bool have_row = qb < nQB;

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Gp = (const uint16_t*)a.dO + (size_t)b * a.so[0] + (size_t)h * a.so[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* dQp = (uint16_t*)a.dQ + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const int sk_bytes = (int)a.sk[2] * 2, sv_bytes = (int)a.sv[2] * 2;
    const rsrc_t k_rsrc = make_rsrc(Kp, (unsigned)((a.Lk - 1) * sk_bytes + D * 2));
    const rsrc_t v_rsrc = make_rsrc(Vp, (unsigned)((a.Lk - 1) * sv_bytes + D * 2));

    const int brow = (wave & 1) * 32 + n;                    // row inside the block row
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
    float lse2 = row_ok ? lse2_of(a.lse[stat]) : INFINITY;
    float delta = row_ok ? a.delta[stat] : 0.f;
    const float sc = a.scale * kLog2e;
    const long long off = (long long)a.Lk - a.Lq;
    const long long diag = (long long)qrow + off;
    const int k_swz = hh ^ swz_k<D>(n);
    const TrRead tr = make_tr_read<D>(lane);

    f32x16 dqacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;

    // the two tile lists; with a causal mask they end at the last column any row of the pair sees
    const int rA = h * nQB + 2 * qp;
    Merge m;
    m.ia = a.row_ptr[rA];
    m.a1 = a.row_ptr[rA + 1];
    m.ib = m.a1;
    m.b1 = (2 * qp + 1 < nQB) ? a.row_ptr[rA + 2] : m.a1;
    const long long pair_diag = (long long)(2 * qp + 1) * 64 + 63 + off;
    const unsigned words_bytes = (unsigned)m.b1 * 512u;     // never read past the pair's last tile

    auto issue = [&](const Merge& x, int stage) {
        lds_u16* base = lds + stage * STAGE;
        const int k0 = x.key * kBN;
        issue_tile_loads<D, 4, false>(k_rsrc, base, k0, sk_bytes, wave, lane);
        issue_tile_loads<D, 4, true>(k_rsrc, base + TILE, k0, sk_bytes, wave, lane);
        issue_tile_loads<D, 4, false>(v_rsrc, base + 2 * TILE, k0, sv_bytes, wave, lane);
        if (wave == 0 && x.ta >= 0) dma_512(base + 3 * TILE, a.bitmaps, words_bytes, (long long)x.ta * 512, lane);
        if (wave == 2 && x.tb >= 0) dma_512(base + 3 * TILE + 256, a.bitmaps, words_bytes, (long long)x.tb * 512, lane);
    };
    auto live = [&](const Merge& x) {                        // anything left that some row can see?
        return x.key != 0x7fffffff && !(a.causal && (long long)x.key * kBN > pair_diag);
    };

    // first use of the loaded registers before the loop, so that no wait for them lands inside it
    wait_vmem();
    settle<KSTEPS>(qreg);
    settle<KSTEPS>(greg);
    asm volatile("" : "+v"(lse2), "+v"(delta));

    Merge cur = m;
    merge_step(cur, a.col_idx);
    Merge nxt = cur;
    int stage = 0;
    if (live(cur)) issue(cur, 0);
    while (live(cur)) {
        merge_step(nxt, a.col_idx);
        wait_vmem();                                         // the current tile has landed
        __syncthreads();                                     // ... for everybody; the other stage is free
        if (live(nxt)) issue(nxt, stage ^ 1);
        const int t = half ? cur.tb : cur.ta;
        const int k0 = cur.key * kBN;
        if (have_row && t >= 0) {
            uint16_t* base = smem + stage * STAGE;
            uint64_t word = *reinterpret_cast<const uint64_t*>(base + 3 * TILE + half * 256 + brow * 4);
            if (a.causal) {
                const long long lim = diag - k0;
                if (lim < 0) word = 0;
                else if (lim < 63) word &= (2ull << lim) - 1ull;
            }
            f32x16 sacc[2], pacc[2];
            qk_64<D>(base, qreg, n, k_swz, sacc);            // S^T  = K Q^T
            qk_64<D>(base + 2 * TILE, greg, n, k_swz, pacc); // dP^T = V dO^T
            const uint64_t wsh = word >> (4 * hh);
            const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int pos = 8 * (i / 4) + (i % 4);
                    // pruned entries: the exponent's argument is replaced by -inf with a bit-select
                    const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)wbits[kb], pos, 1);
                    const float x = fmaf(sacc[kb][i], sc, -lse2);
                    const float p = __builtin_amdgcn_exp2f(__uint_as_float((__float_as_uint(x) & keep) | (0xff800000u & ~keep)));
                    sacc[kb][i] = p * (pacc[kb][i] - delta); // dS^T
                }
            tr_mm_64<D>(lds + stage * STAGE + TILE, sacc, dqacc, tr);   // dQ^T += K^T dS^T
        }
        cur = nxt;
        stage ^= 1;
    }
    __syncthreads();                                         // all wavefronts are done with the tiles
    if (have_row)
        store_rows_bf16<D>(smem + wave * 32 * D, dqacc, a.scale, lane,
                           dQp + (size_t)(qb * 64 + (wave & 1) * 32) * a.sq[2], a.sq[2],
                           a.Lq - (qb * 64 + (wave & 1) * 32));
}

// dK, dV: one workgroup per (example, head, pair of block columns); wavefronts 0,1 own the 64 keys
// of the first block column, wavefronts 2,3 those of the second.  The tiles of both columns are
// walked together in ascending block-row order through the transposed layout, so a Q/dO tile
// that both need is loaded once.  Two LDS stages, one barrier per tile.
template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dkv_kernel(BwdArgs a, int nQB, int nKB, int nKP)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    // Qk, Qv, dOk, dOv, then 256 B lse, 256 B delta, 512 B words of column A, 512 B words of column B
    constexpr int STAGE = 4 * TILE + 768;
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * STAGE];
    lds_u16* lds = (lds_u16*)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;
    const int half = wave >> 1;

    const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int kp = bid % nKP;                                // early causal columns (most tiles) first
    const int h = (bid / nKP) % a.H;
    const int b = bid / (nKP * a.H);
    const int kb = 2 * kp + half;
    const bool have_col = kb < nKB;

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Gp = (const uint16_t*)a.dO + (size_t)b * a.so[0] + (size_t)h * a.so[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* dKp = (uint16_t*)a.dK + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    uint16_t* dVp = (uint16_t*)a.dV + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    const int sq_bytes = (int)a.sq[2] * 2, so_bytes = (int)a.so[2] * 2;
    const rsrc_t q_rsrc = make_rsrc(Qp, (unsigned)((a.Lq - 1) * sq_bytes + D * 2));
    const rsrc_t g_rsrc = make_rsrc(Gp, (unsigned)((a.Lq - 1) * so_bytes + D * 2));
    const size_t stat_base = ((size_t)b * a.H + h) * a.Lq;
    const unsigned stat_bytes = (unsigned)a.Lq * 4u;         // rows >= Lq read as zeros

    const int key = kb * 64 + (wave & 1) * 32 + n;
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
    const int kcol = (wave & 1) * 32 + n;                    // this lane's key inside its tile

    f32x16 dkacc[DBLK], dvacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            dkacc[db][i] = 0.f;
            dvacc[db][i] = 0.f;
        }

    const int cA = h * nKB + 2 * kp;
    Merge m;
    m.ia = a.col_ptr[cA];
    m.a1 = a.col_ptr[cA + 1];
    m.ib = m.a1;
    m.b1 = (2 * kp + 1 < nKB) ? a.col_ptr[cA + 2] : m.a1;
    const unsigned words_bytes = (unsigned)a.row_ptr[a.H * nQB] * 512u;

    auto issue = [&](const Merge& x, int stage) {
        lds_u16* base = lds + stage * STAGE;
        const int q0 = x.key * 64;
        issue_tile_loads<D, 4, false>(q_rsrc, base, q0, sq_bytes, wave, lane);
        issue_tile_loads<D, 4, true>(q_rsrc, base + TILE, q0, sq_bytes, wave, lane);
        issue_tile_loads<D, 4, false>(g_rsrc, base + 2 * TILE, q0, so_bytes, wave, lane);
        issue_tile_loads<D, 4, true>(g_rsrc, base + 3 * TILE, q0, so_bytes, wave, lane);
        lds_u16* st = base + 4 * TILE;
        if (wave == 1 && lane < 16) {                        // 64 floats = 16 lanes x 16 bytes
            load16_to_lds(lds_addr_of(st), lane * 16, make_rsrc(a.lse + stat_base, stat_bytes), q0 * 4);
        }
        if (wave == 3 && lane < 16) {
            load16_to_lds(lds_addr_of(st + 128), lane * 16, make_rsrc(a.delta + stat_base, stat_bytes), q0 * 4);
        }
        if (wave == 0 && x.ta >= 0)
            dma_512(st + 256, a.bitmaps, words_bytes, (long long)a.tile_idx[x.ta] * 512, lane);
        if (wave == 2 && x.tb >= 0)
            dma_512(st + 512, a.bitmaps, words_bytes, (long long)a.tile_idx[x.tb] * 512, lane);
    };
    // a tile is hidden from every query of its block row when the column starts beyond the row's diagonal
    auto live = [&](const Merge& x) { return x.key != 0x7fffffff; };

    wait_vmem();
    settle<KSTEPS>(kreg);
    settle<KSTEPS>(vreg);

    Merge cur = m;
    merge_step(cur, a.row_idx);
    Merge nxt = cur;
    int stage = 0;
    if (live(cur)) issue(cur, 0);
    while (live(cur)) {
        merge_step(nxt, a.row_idx);
        wait_vmem();
        __syncthreads();
        if (live(nxt)) issue(nxt, stage ^ 1);
        const int ci = half ? cur.tb : cur.ta;
        const int q0 = cur.key * 64;
        const bool hidden = a.causal && (long long)kb * 64 > (long long)q0 + 63 + off;
        if (have_col && ci >= 0 && !hidden) {
            uint16_t* base = smem + stage * STAGE;
            const float* s_lse = reinterpret_cast<const float*>(base + 4 * TILE);
            const float* s_delta = reinterpret_cast<const float*>(base + 4 * TILE + 128);
            const uint64_t* s_word = reinterpret_cast<const uint64_t*>(base + 4 * TILE + 256 + half * 256);
            f32x16 sacc[2], pacc[2];
            qk_64<D>(base, kreg, n, k_swz, sacc);            // S  = Q K^T   (rows: queries, lane: key)
            qk_64<D>(base + 2 * TILE, vreg, n, k_swz, pacc); // dP = dO V^T
            const bool diag_tile = a.causal && (long long)kb * 64 + 63 > (long long)q0 + off;
#pragma unroll
            for (int qblk = 0; qblk < 2; ++qblk)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int r0 = 32 * qblk + 8 * g + 4 * hh;   // 4 consecutive query rows
                    const float4 l4 = *reinterpret_cast<const float4*>(&s_lse[r0]);
                    const float4 d4 = *reinterpret_cast<const float4*>(&s_delta[r0]);
                    const float le[4] = {l4.x, l4.y, l4.z, l4.w}, de[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = 4 * g + e;
                        bool kept = (s_word[r0 + e] >> kcol) & 1ull;
                        if (diag_tile) kept = kept && (long long)kb * 64 + kcol <= (long long)q0 + r0 + e + off;
                        const float p = kept ? __builtin_amdgcn_exp2f(fmaf(sacc[qblk][i], sc, -le[e] * kLog2e)) : 0.f;
                        sacc[qblk][i] = p;                   // P
                        pacc[qblk][i] = p * (pacc[qblk][i] - de[e]);   // dS
                    }
                }
            tr_mm_64<D>(lds + stage * STAGE + 3 * TILE, sacc, dvacc, tr);   // dV^T += dO^T P
            tr_mm_64<D>(lds + stage * STAGE + TILE, pacc, dkacc, tr);       // dK^T += Q^T dS
        }
        cur = nxt;
        stage ^= 1;
    }
    __syncthreads();                                         // all wavefronts are done with the tiles
    if (have_col) {
        const int krow0 = kb * 64 + (wave & 1) * 32;
        uint16_t* stg = smem + wave * 32 * D;
        store_rows_bf16<D>(stg, dkacc, a.scale, lane, dKp + (size_t)krow0 * a.sk[2], a.sk[2], a.Lk - krow0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the staging area is reused
        store_rows_bf16<D>(stg, dvacc, 1.0f, lane, dVp + (size_t)krow0 * a.sv[2], a.sv[2], a.Lk - krow0);
    }
}

template <int D>
hipError_t launch_d(const BwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + 63) / 64, nKB = (a.Lk + 63) / 64;
    const int nQP = (nQB + 1) / 2, nKP = (nKB + 1) / 2;
    const long long rows = (long long)a.B * a.H * a.Lq;
    const long long dthreads = rows * (D / 8);
    hipLaunchKernelGGL(bwd_delta_kernel<D>, dim3((unsigned)((dthreads + 255) / 256)), dim3(256), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.sched.cnt) {
        e = launch_bwd_sched(a, true, false, stream);
    } else {
        hipLaunchKernelGGL(bwd_dq_kernel<D>, dim3((unsigned)(a.B * a.H * nQP)), dim3(256), 0, stream, a, nQB, nQP);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    if (a.csched.cnt) return launch_bwd_sched(a, false, true, stream);
    hipLaunchKernelGGL(bwd_dkv_kernel<D>, dim3((unsigned)(a.B * a.H * nKP)), dim3(256), 0, stream, a, nQB, nKB, nKP);
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
