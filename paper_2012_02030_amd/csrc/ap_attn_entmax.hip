// Masked attention forward with the 1.5-entmax normaliser (Section 6: the experiments are
// repeated with 1.5-entmax in place of softmax, together with the pruning mask).
//
// With x_j = scale * <q, k_j> / 2 over the kept, visible keys of a query, 1.5-entmax is
//     p_j = [x_j - tau]_+^2,   tau such that sum_j p_j = 1
// (the optimality conditions of its defining problem).  Unlike softmax this needs a per-row
// threshold before any probability is known, so a workgroup sweeps its block row's tiles
// several times, recomputing S^T = K Q^T on the matrix cores each time (the scores of a long row
// do not fit on chip, and writing them out would cost more than recomputing them):
//
//   sweep 1     row maximum m and the number n of kept visible keys
//   sweeps 2..  with y = x - m <= 0, d = [y - tau]_+: the norm |d| and the sum g of d, and a Newton
//               step on h(tau) = |d| - 1:  tau += (|d| - 1) |d| / g.  h is convex and decreasing
//               with its root in [-1, 0); started at -1 (where h >= 0 because the maximum
//               contributes 1) the steps increase monotonically to the root and never pass it.
//               The norm is much closer to linear than its square, which saves about half of
//               the sweeps.  A row is done when | |d|^2 - 1 | <= 1e-5 at its tau, or after the
//               step taken from a tau with | |d|^2 - 1 | <= 1e-2: the steps converge quadratically,
//               so that step leaves a residual of a few 1e-5 at most (the output is divided by
//               the actual sum of P in any case) and the sweep that would only confirm it is
//               saved.  The block row sweeps until all its rows are done.
//   last sweep  P = [y - tau]_+^2, O^T += V^T P^T, O / sum P.
//
// Same operand layouts, LDS swizzles and LDS-direct loads as the softmax kernel; walks the
// layout's tiles or, if given, the entries of its visit schedule; 64x64 tiles, two LDS stages of K (one barrier per tile) in the threshold sweeps.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"
#include "ap_mfma_common.h"

namespace ap {

namespace {

using namespace mfma;

constexpr float kEntmaxTol = 1e-5f;          // on sum p - 1
constexpr float kEntmaxEarly = 1e-2f;        // residual from which one more step is taken unconfirmed
constexpr int kEntmaxMaxIter = 60;
constexpr int kEntmaxSchedEntries = 64;      // a block row with more schedule entries walks the layout instead
constexpr int kEntmaxGathered = 16;          // ... or with more gathered entries among them

template <int D>
__global__ __launch_bounds__(128, 2) void entmax15_fwd_kernel(FwdArgs a, float* tau_out, int nQB)
{
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    constexpr int STAGE = TILE + 256;                        // a K (or V) tile and 64 bitmap words
    constexpr int RPI = 64 / (D / 8);                        // tile rows per load instruction
    constexpr int NLOAD = (D / 8) / 2;                       // load instructions per wavefront and tile
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * STAGE];
    __shared__ int32_t s_cols[kEntmaxGathered][64];          // gather keys of the block row's gathered entries
    lds_u16* lds = (lds_u16*)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;

    const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int qb = nQB - 1 - (bid % nQB);                    // long causal rows first
    const int h = (bid / nQB) % a.H;
    const int b = bid / (nQB * a.H);

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* Op = (uint16_t*)a.O + (size_t)b * a.so[0] + (size_t)h * a.so[1];
    const int sk_bytes = (int)a.sk[2] * 2, sv_bytes = (int)a.sv[2] * 2;
    const rsrc_t k_rsrc = make_rsrc(Kp, (unsigned)((a.Lk - 1) * sk_bytes + D * 2));
    const rsrc_t v_rsrc = make_rsrc(Vp, (unsigned)((a.Lk - 1) * sv_bytes + D * 2));

    const int brow = wave * 32 + n;
    const int qrow = qb * 64 + brow;
    const bool row_ok = qrow < a.Lq;
    bf16x8 qreg[KSTEPS];
    {
        const uint16_t* qr = Qp + (size_t)(row_ok ? qrow : a.Lq - 1) * a.sq[2] + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) qreg[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
    }
    const float c = 0.5f * a.scale;                          // x = c * <q, k>
    const long long off = (long long)a.Lk - a.Lq;
    const long long diag = (long long)qrow + off;
    const long long block_diag = (long long)qb * 64 + 63 + off;
    const int k_swz = hh ^ swz_k<D>(n);
    const TrRead tr = make_tr_read<D>(lane);

    const int r = h * nQB + qb;
    const int t0 = a.row_ptr[r];
    int t1 = a.row_ptr[r + 1];
    // With a visit schedule the entries of the block row replace its tiles: runs of 64 consecutive
    // keys or 64 gathered keys, causal limit already folded into their bitmaps.  The gather keys
    // are read every sweep, so they are copied to LDS once.
    bool use_sched = a.sched.cnt != nullptr && a.sched.cnt[r] <= kEntmaxSchedEntries;
    uint64_t gathered = 0;                                   // bit e: entry e of the block row is gathered
    if (use_sched) {
        const int ne = a.sched.cnt[r];
        gathered = __ballot(lane < ne && a.sched.start[t0 + lane] < 0);
        use_sched = __popcll(gathered) <= kEntmaxGathered;
    }
    if (use_sched) {
        t1 = t0 + a.sched.cnt[r];
        int slot = 0;
        for (uint64_t mm = gathered; mm; mm &= mm - 1, ++slot) {
            const int e = __ffsll((long long)mm) - 1;
            if (tid < 64) s_cols[slot][tid] = a.sched.cols[(size_t)(t0 + e) * 64 + tid];
        }
    } else if (a.causal) {                                   // columns ascend: hidden tiles are at the end
        while (t1 > t0 && (long long)a.col_idx[t1 - 1] * kBN > block_diag) --t1;
    }
    const uint64_t* words = use_sched ? a.sched.bitmaps : a.bitmaps;
    const unsigned words_bytes = (unsigned)a.row_ptr[r + 1] * 512u;
    const int g_row = lane / (D / 8);

    wait_vmem();
    settle<KSTEPS>(qreg);

    f32x16 oacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;

    // One sweep over the tiles of the block row; `body(word, sacc, stage)` sees the raw scores of
    // a tile with pruned and hidden entries already replaced by -inf.
    auto sweep = [&](bool with_v, auto&& body) {
        // without V: two stages, the next K tile travels while the current one is used.
        // with V (last sweep only): K in the first buffer, V in the second, loaded per tile.
        auto issue = [&](int t, int stage) {
            lds_u16* base = lds + stage * STAGE;
            const int k0 = use_sched ? a.sched.start[t] : a.col_idx[t] * kBN;
            if (k0 >= 0) {
                issue_tile_loads<D, 2, false>(k_rsrc, base, k0, sk_bytes, wave, lane);
                if (with_v) issue_tile_loads<D, 2, true>(v_rsrc, lds + STAGE, k0, sv_bytes, wave, lane);
            } else {                                         // gathered entry: an empty slot holds Lk (reads zeros)
                int gk[NLOAD];
                const int slot = __popcll(gathered & ((1ull << (t - t0)) - 1ull));
#pragma unroll
                for (int u = 0; u < NLOAD; ++u) gk[u] = s_cols[slot][(wave + 2 * u) * RPI + g_row];
                issue_gather_loads<D, 2, false>(k_rsrc, base, gk, sk_bytes, wave, lane);
                if (with_v) issue_gather_loads<D, 2, true>(v_rsrc, lds + STAGE, gk, sv_bytes, wave, lane);
            }
            if (wave == 0) dma_512(base + TILE, words, words_bytes, (long long)t * 512, lane);
        };
        __syncthreads();                                     // the previous sweep is done with both buffers
        if (!with_v && t0 < t1) issue(t0, 0);
        int stage = 0;
        for (int t = t0; t < t1; ++t) {
            if (with_v) {
                __syncthreads();                             // the previous tile is consumed
                issue(t, 0);
            }
            wait_vmem();
            __syncthreads();
            if (!with_v && t + 1 < t1) issue(t + 1, stage ^ 1);
            uint16_t* base = smem + stage * STAGE;
            uint64_t word = *reinterpret_cast<const uint64_t*>(base + TILE + brow * 4);
            if (a.causal && !use_sched) {
                const long long lim = diag - (long long)a.col_idx[t] * kBN;
                if (lim < 0) word = 0;
                else if (lim < 63) word &= (2ull << lim) - 1ull;
            }
            if (__ballot(word != 0) != 0) {
                f32x16 sacc[2];
                qk_64<D>(base, qreg, n, k_swz, sacc);
                const uint64_t wsh = word >> (4 * hh);
                const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int pos = 8 * (i / 4) + (i % 4);
                        const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)wbits[kb], pos, 1);
                        sacc[kb][i] = __uint_as_float((__float_as_uint(sacc[kb][i]) & keep) | (0xff800000u & ~keep));
                    }
                body(word, sacc);
            }
            if (!with_v) stage ^= 1;
        }
    };
    auto both_halves_max = [&](float v) {
        const auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        return fmaxf(__uint_as_float(s[0]), __uint_as_float(s[1]));
    };
    auto both_halves_sum = [&](float v) {
        const auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        return __uint_as_float(s[0]) + __uint_as_float(s[1]);
    };

    // ---- sweep 1: row maximum and number of kept visible keys
    float m = -INFINITY;
    int nkept = 0;
    sweep(false, [&](uint64_t word, f32x16* sacc) {
        nkept += __popcll(word);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) m = fmaxf(m, sacc[kb][i]);
    });
    m = both_halves_max(m);
    const bool empty = nkept == 0;                           // both halves counted the same words
    const float mc = empty ? 0.f : m * c;

    // ---- Newton sweeps for tau (relative to the row maximum: the root lies in [-1, 0))
    float tau = -1.f;
    bool done = empty;
    for (int iter = 0; iter < kEntmaxMaxIter; ++iter) {
        if (__syncthreads_or(done ? 0 : 1) == 0) break;      // every row of the block row has its tau
        float g1 = 0.f, g2 = 0.f;
        sweep(false, [&](uint64_t, f32x16* sacc) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float d = fmaxf(fmaf(sacc[kb][i], c, -mc) - tau, 0.f);   // -inf -> 0
                    g1 += d;
                    g2 = fmaf(d, d, g2);
                }
        });
        g1 = both_halves_sum(g1);
        g2 = both_halves_sum(g2);
        if (!done) {
            const float f = g2 - 1.0f;
            if (fabsf(f) <= kEntmaxTol || g1 <= 0.f) {
                done = true;
            } else {
                const float nd = sqrtf(g2);
                tau = fminf(fmaxf(tau + (nd - 1.0f) * nd / g1, -1.0f), 0.f);
                done = fabsf(f) <= kEntmaxEarly;             // this step is the last one
            }
        }
    }

    // ---- last sweep: probabilities and output
    float psum = 0.f;
    sweep(true, [&](uint64_t, f32x16* sacc) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float d = fmaxf(fmaf(sacc[kb][i], c, -mc) - tau, 0.f);
                const float p = d * d;
                sacc[kb][i] = p;
                psum += p;
            }
        tr_mm_64<D>(lds + STAGE, sacc, oacc, tr);
    });
    psum = both_halves_sum(psum);
    const float inv = (!empty && psum > 0.f) ? 1.0f / psum : 0.f;

    __syncthreads();                                         // all wavefronts are done with the tiles
    store_rows_bf16<D>(smem + wave * 32 * D, oacc, inv, lane, Op + (size_t)(qb * 64 + wave * 32) * a.so[2],
                       a.so[2], a.Lq - (qb * 64 + wave * 32));
    if (tau_out && row_ok && hh == 0)
        tau_out[((size_t)b * a.H + h) * a.Lq + qrow] = empty ? INFINITY : mc + tau;
}

template <int D>
hipError_t launch_d(const FwdArgs& a, float* tau_out, hipStream_t stream)
{
    const int nQB = (a.Lq + 63) / 64;
    hipLaunchKernelGGL(entmax15_fwd_kernel<D>, dim3((unsigned)(a.B * a.H * nQB)), dim3(128), 0, stream, a,
                       tau_out, nQB);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_entmax15_fwd(const FwdArgs& a, float* tau_out, hipStream_t stream)
{
    switch (a.D) {
        case 32: return launch_d<32>(a, tau_out, stream);
        case 64: return launch_d<64>(a, tau_out, stream);
        case 128: return launch_d<128>(a, tau_out, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ap
