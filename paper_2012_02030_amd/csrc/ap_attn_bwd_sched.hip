// Backward pass over visit schedules: the same arithmetic as ap_attn_bwd.hip, but dQ walks the
// entries of the row schedule (runs of 64 consecutive keys or 64 gathered keys per block row) and
// dK, dV walk the entries of the column schedule (runs of 64 consecutive queries or 64 gathered
// queries per block column), so the backward pass skips what the forward pass skips.  Causal
// limits are folded into the entry bitmaps by the schedule builders.
//
// One workgroup of two wavefronts per block row (dQ) or block column (dK, dV).  Every tile is
// stored once in LDS, with a swizzle that suits both the row-wise reads (scores) and the
// transposing reads (gradient products).  Two LDS stages: the next entry's tiles travel while the
// current entry is computed; the metadata of the entry after that (start, gather indices, bitmap
// words, per-query statistics) is fetched into registers in the same step.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"
#include "ap_mfma_common.h"

namespace ap {

namespace {

using namespace mfma;

// What the kernels compute per entry.  SOFTMAX: P = exp(s - lse), dS = P (dP - delta) with the
// per-query statistics lse and delta = <dO, O>.  ENTMAX15 (the 1.5-entmax normaliser of Section 6):
// u = [s / 2 - tau]_+, P = u^2, dS = u (dP - gbar) with the per-query statistics tau (from the
// forward pass) and gbar = sum_j u_j dP_j / sum_j u_j, which GBAR, a dQ-shaped pass that stops
// before the last product, computes first.  For the two entmax modes BwdArgs::lse holds tau and
// BwdArgs::delta holds gbar.
enum { SOFTMAX = 0, ENTMAX15 = 1, GBAR = 2 };

__device__ __forceinline__ float lse2_of(float lse) { return lse == -INFINITY ? INFINITY : lse * kLog2e; }

template <int D, int MODE>
__global__ __launch_bounds__(128, D == 128 ? 1 : 2) void bwd_dq_sched_kernel(BwdArgs a, int nQB)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    constexpr int RPI = 64 / (D / 8);
    constexpr int NLOAD = (D / 8) / 2;
    constexpr int STAGE = 2 * TILE;                          // K rows, V rows
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * STAGE];
    lds_u16* lds = (lds_u16*)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;
    const int g_row = lane / (D / 8);
    // A zero the compiler cannot see through.  Indexing with it turns the per-entry load of a
    // start into a vector load: a scalar load inside the loop would make every later wait for an
    // LDS read (same counter, scalar loads return out of order) wait for memory as well.
    int vzero = 0;
    asm volatile("" : "+v"(vzero));

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
    // SOFTMAX: base-2 log-sum-exp and delta; entmax modes: tau (+inf for a query without keys) and gbar
    float lse2 = row_ok ? (MODE == SOFTMAX ? lse2_of(a.lse[stat]) : a.lse[stat]) : INFINITY;
    float delta = row_ok && MODE != GBAR ? a.delta[stat] : 0.f;
    const float sc = MODE == SOFTMAX ? a.scale * kLog2e : a.scale * 0.5f;
    float num = 0.f, den = 0.f;                              // GBAR: this lane's share of sum u dP and sum u
    const int k_swz = hh ^ swz_u<D>(n);
    const TrReadU<D> tr = make_tr_read_u<D>(lane);

    f32x16 dqacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;

    const int r = h * nQB + qb;
    const int t0 = a.row_ptr[r];
    const int t1 = t0 + a.sched.cnt[r];

    // metadata of an entry: where it starts (or -1), gather key `lane` (read for every entry,
    // used by gathered ones only) and this lane's bitmap word: three loads per entry
    struct Meta {
        int start;
        int key;
        uint64_t word;
    };
    auto fetch = [&](int t, Meta& m) {
        m.start = a.sched.start[t + vzero];                  // a vector load: see vzero
        m.key = a.sched.cols[(size_t)t * 64 + lane];
        m.word = a.sched.bitmaps[(size_t)t * 64 + brow];     // causal limit folded in
    };
    auto issue = [&](const Meta& m, int stage) {
        lds_u16* base = lds + stage * STAGE;
        const int start = __builtin_amdgcn_readfirstlane(m.start);
        if (start >= 0) {
            issue_tile_loads<D, 2, SWZ_BOTH>(k_rsrc, base, start, sk_bytes, wave, lane);
            issue_tile_loads<D, 2, SWZ_BOTH>(v_rsrc, base + TILE, start, sv_bytes, wave, lane);
        } else {
            int gk[NLOAD];                                   // keys of the rows this lane loads
#pragma unroll
            for (int u = 0; u < NLOAD; ++u) gk[u] = __shfl(m.key, (wave + 2 * u) * RPI + g_row, 64);
            issue_gather_loads<D, 2, SWZ_BOTH>(k_rsrc, base, gk, sk_bytes, wave, lane);
            issue_gather_loads<D, 2, SWZ_BOTH>(v_rsrc, base + TILE, gk, sv_bytes, wave, lane);
        }
    };

    Meta cur, nxt;
    if (t0 < t1) {
        fetch(t0, cur);
        issue(cur, 0);
        nxt = cur;
        if (t0 + 1 < t1) fetch(t0 + 1, nxt);
    }
    // first use of the loaded registers before the loop, so that no wait for them lands inside it
    wait_vmem();
    settle<KSTEPS>(qreg);
    settle<KSTEPS>(greg);
    asm volatile("" : "+v"(lse2), "+v"(delta));

    int stage = 0;
    for (int t = t0; t < t1; ++t) {
        wait_vmem();                                         // entry t and the metadata of t + 1 have landed
        __syncthreads();                                     // ... for everybody; the other stage is free
        const uint64_t word = cur.word;
        if (t + 1 < t1) {
            issue(nxt, stage ^ 1);
            cur = nxt;
            if (t + 2 < t1) fetch(t + 2, nxt);
        }
        if (__ballot(word != 0) != 0) {
            uint16_t* base = smem + stage * STAGE;
            f32x16 sacc[2], pacc[2];
            qk_64<D>(base, qreg, n, k_swz, sacc);            // S^T  = K Q^T
            qk_64<D>(base + TILE, greg, n, k_swz, pacc);     // dP^T = V dO^T
            const uint64_t wsh = word >> (4 * hh);
            const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int pos = 8 * (i / 4) + (i % 4);
                    const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)wbits[kb], pos, 1);
                    const float x = fmaf(sacc[kb][i], sc, -lse2);
                    if (MODE == SOFTMAX) {
                        const float p = __builtin_amdgcn_exp2f(__uint_as_float((__float_as_uint(x) & keep) | (0xff800000u & ~keep)));
                        sacc[kb][i] = p * (pacc[kb][i] - delta);   // dS^T
                    } else {
                        const float u = fmaxf(__uint_as_float(__float_as_uint(x) & keep), 0.f);   // pruned: 0
                        if (MODE == GBAR) {
                            num = fmaf(u, pacc[kb][i], num);
                            den += u;
                        } else {
                            sacc[kb][i] = u * (pacc[kb][i] - delta);   // dS^T
                        }
                    }
                }
            if (MODE != GBAR) tr_mm_64_u<D>(lds + stage * STAGE, sacc, dqacc, tr);   // dQ^T += K^T dS^T
        }
        stage ^= 1;
    }
    if (MODE == GBAR) {                                      // the two half-wavefronts hold different keys
        num += __shfl_xor(num, 32, 64);
        den += __shfl_xor(den, 32, 64);
        if (row_ok && hh == 0) a.delta[stat] = den > 0.f ? num / den : 0.f;
        return;
    }
    __syncthreads();                                         // all wavefronts are done with the tiles
    store_rows_bf16<D>(smem + wave * 32 * D, dqacc, a.scale, lane,
                       dQp + (size_t)(qb * 64 + wave * 32) * a.sq[2], a.sq[2], a.Lq - (qb * 64 + wave * 32));
}

// Two wavefronts per SIMD where the registers allow it without spilling (the 1.5-entmax form at
// D = 64 needs a few more than 256).
template <int D, int NORM>
__global__ __launch_bounds__(128, (D == 128 || (D == 64 && NORM == 1)) ? 1 : 2) void bwd_dkv_sched_kernel(BwdArgs a, int nKB)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    constexpr int RPI = 64 / (D / 8);
    constexpr int NLOAD = (D / 8) / 2;
    constexpr int STAGE = 2 * TILE;                          // Q rows, dO rows
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * STAGE];
    __shared__ __attribute__((aligned(16))) float s_lse2[2][64];
    __shared__ __attribute__((aligned(16))) float s_delta[2][64];
    __shared__ __attribute__((aligned(16))) uint32_t s_half[2][2][64];   // bitmap words: low halves, high halves
    lds_u16* lds = (lds_u16*)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;
    const int g_row = lane / (D / 8);
    // A zero the compiler cannot see through.  Indexing with it turns the per-entry load of a
    // start into a vector load: a scalar load inside the loop would make every later wait for an
    // LDS read (same counter, scalar loads return out of order) wait for memory as well.
    int vzero = 0;
    asm volatile("" : "+v"(vzero));

    // Which (example, head) pair and which position of the head's visiting order this workgroup
    // takes.  Every XCD gets a contiguous range of pairs (they share Q and dO rows in its L2); when
    // the pairs divide evenly over the 8 XCDs, the heavy columns of all pairs of the range come
    // first, so that the longest workgroups start at once, then the other columns pair by pair.
    const int32_t* order = a.csched.cnt + (size_t)a.H * nKB;
    const int32_t* n_heavy = order + (size_t)a.H * nKB;
    const int NP = a.B * a.H;
    int pair, idx;
    if (NP % 8 == 0 && NP / 8 <= 64) {
        // lane p looks at pair P0 + p: one load and two wave-wide prefix sums instead of a chain of
        // dependent scalar loads
        const int PP = NP / 8, P0 = (blockIdx.x & 7) * PP;
        const int l = blockIdx.x >> 3;
        const int hv = lane < PP ? n_heavy[(P0 + lane) % a.H] : 0;
        const int lt = lane < PP ? nKB - hv : 0;
        int hv_incl = hv, lt_incl = lt;                      // inclusive prefix sums over the lanes
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int x = __shfl_up(hv_incl, o, 64), y = __shfl_up(lt_incl, o, 64);
            if (lane >= o) {
                hv_incl += x;
                lt_incl += y;
            }
        }
        const int hv_total = __shfl(hv_incl, 63, 64);
        const bool in_heavy = l < hv_total;
        const int ll = in_heavy ? l : l - hv_total;
        const int incl = in_heavy ? hv_incl : lt_incl, mine = in_heavy ? hv : lt;
        // the lane whose range [incl - mine, incl) holds ll
        const unsigned long long hit = __ballot(lane < PP && ll >= incl - mine && ll < incl);
        if (hit == 0) return;                                // cannot happen for grid = pairs x columns
        const int p = __ffsll((long long)hit) - 1;           // exactly one lane
        pair = P0 + p;
        idx = ll - (__shfl(incl, p, 64) - __shfl(mine, p, 64)) + (in_heavy ? 0 : __shfl(hv, p, 64));
        pair = __builtin_amdgcn_readfirstlane(pair);
        idx = __builtin_amdgcn_readfirstlane(idx);
    } else {
        const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
        pair = bid / nKB;
        idx = bid % nKB;
    }
    const int h = pair % a.H;
    const int b = pair / a.H;
    const int kb = order[(size_t)h * nKB + idx];

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
    const float sc = NORM == SOFTMAX ? a.scale * kLog2e : a.scale * 0.5f;
    const int k_swz = hh ^ swz_u<D>(n);
    const TrReadU<D> tr = make_tr_read_u<D>(lane);

    f32x16 dkacc[DBLK], dvacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            dkacc[db][i] = 0.f;
            dvacc[db][i] = 0.f;
        }

    const int c = h * nKB + kb;
    const int t0 = a.col_ptr[c];
    const int t1 = t0 + a.csched.cnt[c];

    // metadata of an entry: where it starts (or -1) and gathered query `lane` (read for every
    // entry, used by gathered ones only)
    struct Meta {
        int start;
        int row;
    };
    // per-slot statistics of an entry, fetched by the first 64 threads one step ahead
    struct Stat {
        float lse, delta;
        uint64_t word;
    };
    auto fetch = [&](int t, Meta& m) {
        m.start = a.csched.start[t + vzero];                 // a vector load: see vzero
        m.row = a.csched.cols[(size_t)t * 64 + lane];
    };
    auto fetch_stat = [&](int t, const Meta& m, Stat& s) {
        if (tid < 64) {
            const int q = m.start >= 0 ? m.start + tid : m.row;   // (all lanes hold the same start)
            const int ql = q < a.Lq ? q : a.Lq - 1;
            const float l = a.lse[stat_base + ql], d = a.delta[stat_base + ql];
            s.lse = q < a.Lq ? l : (NORM == SOFTMAX ? -INFINITY : INFINITY);   // lse, or tau
            s.delta = q < a.Lq ? d : 0.f;
            s.word = a.csched.bitmaps[(size_t)t * 64 + tid];
        }
    };
    auto issue = [&](const Meta& m, int stage) {
        lds_u16* base = lds + stage * STAGE;
        const int start = __builtin_amdgcn_readfirstlane(m.start);
        if (start >= 0) {
            issue_tile_loads<D, 2, SWZ_BOTH>(q_rsrc, base, start, sq_bytes, wave, lane);
            issue_tile_loads<D, 2, SWZ_BOTH>(g_rsrc, base + TILE, start, so_bytes, wave, lane);
        } else {
            int gq[NLOAD];                                   // queries of the rows this lane loads
#pragma unroll
            for (int u = 0; u < NLOAD; ++u) gq[u] = __shfl(m.row, (wave + 2 * u) * RPI + g_row, 64);
            issue_gather_loads<D, 2, SWZ_BOTH>(q_rsrc, base, gq, sq_bytes, wave, lane);
            issue_gather_loads<D, 2, SWZ_BOTH>(g_rsrc, base + TILE, gq, so_bytes, wave, lane);
        }
    };

    Meta cur, nxt;
    Stat st;
    st.lse = NORM == SOFTMAX ? -INFINITY : INFINITY;
    st.delta = 0.f;
    st.word = 0;
    if (t0 < t1) {
        fetch(t0, cur);
        issue(cur, 0);
        fetch_stat(t0, cur, st);
        nxt = cur;
        if (t0 + 1 < t1) fetch(t0 + 1, nxt);
    }
    wait_vmem();
    settle<KSTEPS>(kreg);
    settle<KSTEPS>(vreg);

    int stage = 0;
    for (int t = t0; t < t1; ++t) {
        wait_vmem();                                         // entry t, its statistics and the metadata of t + 1
        if (tid < 64) {
            s_lse2[stage][tid] = NORM == SOFTMAX ? lse2_of(st.lse) : st.lse;
            s_delta[stage][tid] = st.delta;
            s_half[stage][0][tid] = (uint32_t)st.word;
            s_half[stage][1][tid] = (uint32_t)(st.word >> 32);
        }
        __syncthreads();                                     // ... for everybody; the other stage is free
        if (t + 1 < t1) {
            issue(nxt, stage ^ 1);
            fetch_stat(t + 1, nxt, st);
            if (t + 2 < t1) fetch(t + 2, nxt);
        }
        uint16_t* base = smem + stage * STAGE;
        f32x16 sacc[2], pacc[2];
        qk_64<D>(base, kreg, n, k_swz, sacc);                // S  = Q K^T   (rows: queries, lane: key)
        qk_64<D>(base + TILE, vreg, n, k_swz, pacc);         // dP = dO V^T
        const uint32_t* halves = &s_half[stage][wave][0];    // this wavefront's 32 keys: bit n of these
#pragma unroll
        for (int qblk = 0; qblk < 2; ++qblk)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int r0 = 32 * qblk + 8 * g + 4 * hh;   // 4 consecutive query slots
                const float4 l4 = *reinterpret_cast<const float4*>(&s_lse2[stage][r0]);
                const float4 d4 = *reinterpret_cast<const float4*>(&s_delta[stage][r0]);
                const uint4 w4 = *reinterpret_cast<const uint4*>(&halves[r0]);
                const float le[4] = {l4.x, l4.y, l4.z, l4.w}, de[4] = {d4.x, d4.y, d4.z, d4.w};
                const uint32_t we[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * g + e;
                    // pruned entries: the exponent's argument is replaced by -inf with a bit-select
                    const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)we[e], n, 1);
                    const float x = fmaf(sacc[qblk][i], sc, -le[e]);
                    if (NORM == SOFTMAX) {
                        const float p = __builtin_amdgcn_exp2f(__uint_as_float((__float_as_uint(x) & keep) | (0xff800000u & ~keep)));
                        sacc[qblk][i] = p;                   // P
                        pacc[qblk][i] = p * (pacc[qblk][i] - de[e]);   // dS
                    } else {
                        const float u = fmaxf(__uint_as_float(__float_as_uint(x) & keep), 0.f);   // pruned: 0
                        sacc[qblk][i] = u * u;               // P
                        pacc[qblk][i] = u * (pacc[qblk][i] - de[e]);   // dS
                    }
                }
            }
        tr_mm_64_u<D>(lds + stage * STAGE + TILE, sacc, dvacc, tr);   // dV^T += dO^T P
        tr_mm_64_u<D>(lds + stage * STAGE, pacc, dkacc, tr);          // dK^T += Q^T dS
        stage ^= 1;
    }
    __syncthreads();                                         // all wavefronts are done with the tiles
    const int krow0 = kb * 64 + wave * 32;
    uint16_t* stg = smem + wave * 32 * D;
    store_rows_bf16<D>(stg, dkacc, a.scale, lane, dKp + (size_t)krow0 * a.sk[2], a.sk[2], a.Lk - krow0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the staging area is reused
    store_rows_bf16<D>(stg, dvacc, 1.0f, lane, dVp + (size_t)krow0 * a.sv[2], a.sv[2], a.Lk - krow0);
}

template <int D>
hipError_t launch_d(const BwdArgs& a, bool dq, bool dkv, hipStream_t stream)
{
    const int nQB = (a.Lq + 63) / 64, nKB = (a.Lk + 63) / 64;
    const dim3 qgrid((unsigned)(a.B * a.H * nQB)), kgrid((unsigned)(a.B * a.H * nKB));
    if (a.entmax) {                                          // gbar first, then the two gradient kernels
        hipLaunchKernelGGL((bwd_dq_sched_kernel<D, GBAR>), qgrid, dim3(128), 0, stream, a, nQB);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((bwd_dq_sched_kernel<D, ENTMAX15>), qgrid, dim3(128), 0, stream, a, nQB);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((bwd_dkv_sched_kernel<D, ENTMAX15>), kgrid, dim3(128), 0, stream, a, nKB);
        return hipGetLastError();
    }
    if (dq) {
        hipLaunchKernelGGL((bwd_dq_sched_kernel<D, SOFTMAX>), qgrid, dim3(128), 0, stream, a, nQB);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (dkv) hipLaunchKernelGGL((bwd_dkv_sched_kernel<D, SOFTMAX>), kgrid, dim3(128), 0, stream, a, nKB);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_sched(const BwdArgs& a, bool dq, bool dkv, hipStream_t stream)
{
    switch (a.D) {
        case 32: return launch_d<32>(a, dq, dkv, stream);
        case 64: return launch_d<64>(a, dq, dkv, stream);
        case 128: return launch_d<128>(a, dq, dkv, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ap
