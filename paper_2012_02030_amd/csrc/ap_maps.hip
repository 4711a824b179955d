// Accumulation of attention matrices into the mean attention map (Section 3.2, Eq. (1)).
//
// The attention matrix of one example, A_b = softmax(Q_b K_b^T / sqrt(d_k)), is never stored:
// it would be B*H*Lq*Lk probabilities.  Two kernels instead:
//
//   row_lse_kernel         one workgroup per (example, head, 128 queries): walks all key tiles,
//                          S^T = K Q^T on the matrix cores, keeps the online row maximum and row
//                          sum, and writes the row's log-sum-exp (base 2) to the workspace.
//   map_accumulate_kernel  one workgroup per (head, 128 queries, 128 keys): loops over the
//                          examples, recomputes the scores tile by tile, P = exp2(s - lse), and
//                          sums P in registers; the running map in memory is read and written
//                          once per call, whatever the batch size.
//
// Both use the score layout of the attention kernel: a wavefront owns 32 queries, lane l holds
// query l % 32 and, of each 32-key block, the keys 8*(i/4) + 4*(l/32) + i%4 (i = 0..15).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"
#include "ap_mfma_common.h"

namespace ap {

namespace {

using namespace mfma;

template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void row_lse_kernel(MapArgs a, int nQB)
{
    constexpr int BM = 32 * NW;
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * TILE];
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
    const int sk_bytes = (int)a.sk[2] * 2;
    const rsrc_t k_rsrc = make_rsrc(Kp, (unsigned)((a.Lk - 1) * sk_bytes + D * 2));

    const int qrow = qb * BM + wave * 32 + n;
    const bool row_ok = qrow < a.Lq;
    bf16x8 qreg[KSTEPS];
    {
        const uint16_t* qr = Qp + (size_t)(row_ok ? qrow : a.Lq - 1) * a.sq[2] + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            qreg[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
    }
    const long long off = (long long)a.Lk - a.Lq;
    const long long diag = (long long)qrow + off;            // last visible key if causal
    int nkt = (a.Lk + 63) / 64;
    if (a.causal) {
        const long long block_diag = (long long)qb * BM + (BM - 1) + off;
        nkt = (int)min((long long)nkt, block_diag / 64 + 1);
    }
    const int k_swz = hh ^ swz_k<D>(n);
    const float sc = a.scale * kLog2e;
    float m = -INFINITY, lsum = 0.f;

    wait_vmem();
    settle<KSTEPS>(qreg);
    issue_tile_loads<D, NW, false>(k_rsrc, lds, 0, sk_bytes, wave, lane);
    for (int kt = 0; kt < nkt; ++kt) {
        wait_vmem();                                         // tile kt has landed
        __syncthreads();                                     // ... for everybody; tile kt-1 is consumed
        if (kt + 1 < nkt)
            issue_tile_loads<D, NW, false>(k_rsrc, lds + ((kt + 1) & 1) * TILE, (kt + 1) * 64,
                                           sk_bytes, wave, lane);
        f32x16 sacc[2];
        qk_64<D>(smem + (kt & 1) * TILE, qreg, n, k_swz, sacc);

        // keys of this tile that exist and that this query may see: a prefix of the tile
        const long long k0 = (long long)kt * 64;
        long long lim = (long long)a.Lk - k0;
        if (a.causal) lim = min(lim, diag - k0 + 1);
        float tmax = -INFINITY;
        if (__ballot(lim < 64) == 0) {                       // whole tile visible to the whole wavefront
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sacc[kb][i]);
        } else {
            const uint64_t word = lim >= 64 ? ~0ull : (lim <= 0 ? 0ull : (1ull << lim) - 1ull);
            const uint64_t wsh = word >> (4 * hh);
            const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int pos = 8 * (i / 4) + (i % 4);
                    const float sv = ((wbits[kb] >> pos) & 1u) ? sacc[kb][i] : -INFINITY;
                    sacc[kb][i] = sv;
                    tmax = fmaxf(tmax, sv);
                }
        }
        {
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
            tmax = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
        }
        const float m_new = fmaxf(m, tmax);
        const float msc = (m_new == -INFINITY) ? 0.f : m_new * sc;
        const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m * sc - msc);
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) psum += __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], sc, -msc));
        lsum = lsum * alpha + psum;
        m = m_new;
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lsum), __float_as_uint(lsum), false, false);
        lsum = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    if (row_ok && hh == 0)
        a.lse2[((size_t)b * a.H + h) * a.Lq + qrow] =
            (m == -INFINITY) ? -INFINITY : fmaf(m, sc, __log2f(lsum));
}

// One workgroup: 32*NW queries x KT*64 keys of one head.  The Q rows of an example are loaded
// once for all KT key tiles, every K tile serves all NW wavefronts, and the KT partial maps stay
// in registers over the examples.
template <int D, int NW, int KT>
__global__ __launch_bounds__(64 * NW) void map_accumulate_kernel(MapArgs a, int nQB, int nKG)
{
    constexpr int BM = 32 * NW;
    constexpr int TILE = kBN * D;
    constexpr int KSTEPS = D / 16;
    constexpr int OUT_LD = 68;                               // floats per staged output row (16-byte rows)
    constexpr int OUT_ELEMS = BM * OUT_LD * 2;               // in 2-byte units
    constexpr int SMEM = 2 * TILE > OUT_ELEMS ? 2 * TILE : OUT_ELEMS;
    __shared__ __attribute__((aligned(1024))) uint16_t smem[SMEM];
    lds_u16* lds = (lds_u16*)smem;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;

    const int bid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int kg = bid % nKG;
    const int qb = (bid / nKG) % nQB;
    const int h = bid / (nKG * nQB);
    const long long off = (long long)a.Lk - a.Lq;
    const int key0 = kg * (KT * 64);                         // first key of this workgroup
    int n_sub = min(KT, (a.Lk - key0 + 63) / 64);            // key tiles that exist ...
    if (a.causal) {                                          // ... and that some query of the block sees
        const long long block_diag = (long long)qb * BM + (BM - 1) + off;
        if (block_diag < key0) return;
        n_sub = (int)min((long long)n_sub, (block_diag - key0) / 64 + 1);
    }

    const int qrow = qb * BM + wave * 32 + n;
    const int qload = qrow < a.Lq ? qrow : a.Lq - 1;
    const int sk_bytes = (int)a.sk[2] * 2;
    const unsigned k_bytes = (unsigned)((a.Lk - 1) * sk_bytes + D * 2);
    const int k_swz = hh ^ swz_k<D>(n);
    const float sc = a.scale * kLog2e;

    auto q_row = [&](int b) {
        return (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1] +
               (size_t)qload * a.sq[2] + 8 * hh;
    };
    auto issue_k = [&](int b, int sub, int stage) {
        const rsrc_t rs = make_rsrc((const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1], k_bytes);
        issue_tile_loads<D, NW, false>(rs, lds + stage * TILE, key0 + sub * 64, sk_bytes, wave, lane);
    };

    f32x16 acc[KT][2];
#pragma unroll
    for (int sub = 0; sub < KT; ++sub)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[sub][kb][i] = 0.f;

    bf16x8 qcur[KSTEPS];
    float lcur, lnext = 0.f;
    {
        const uint16_t* qr = q_row(0);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) qcur[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
        lcur = a.lse2[(size_t)h * a.Lq + qload];
        issue_k(0, 0, 0);
    }
    int stage = 0;
    for (int b = 0; b < a.B; ++b) {
#pragma unroll
        for (int sub = 0; sub < KT; ++sub) {
            if (sub >= n_sub) continue;                      // uniform over the workgroup
            wait_vmem();                                     // this K tile (and new Q rows) have landed
            settle<KSTEPS>(qcur);
            asm volatile("" : "+v"(lnext), "+v"(lcur));
            if (sub == 0 && b > 0) lcur = lnext;
            __syncthreads();                                 // ... for everybody; the other stage is free
            const bool last = sub + 1 == n_sub;
            if (!last) issue_k(b, sub + 1, stage ^ 1);       // the next tile travels under the arithmetic
            else if (b + 1 < a.B) issue_k(b + 1, 0, stage ^ 1);
            f32x16 sacc[2];
            qk_64<D>(smem + stage * TILE, qcur, n, k_swz, sacc);
            if (last && b + 1 < a.B) {                       // Q rows and lse of the next example
                const uint16_t* qr = q_row(b + 1);
#pragma unroll
                for (int kk = 0; kk < KSTEPS; ++kk) qcur[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
                lnext = a.lse2[((size_t)(b + 1) * a.H + h) * a.Lq + qload];
            }
            // entries outside the map or hidden by causality are computed too (from zero keys or
            // real ones) and dropped when the tile is written
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    acc[sub][kb][i] += __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], sc, -lcur));
            stage ^= 1;
        }
    }

    // transpose through LDS: lanes hold columns of keys per query, memory wants rows of keys
    float* outs = reinterpret_cast<float*>(smem);
    const bool vec_ok = (a.Lk & 3) == 0;                     // then every row of the map starts 16-byte aligned
    const int c4 = (tid & 15) * 4;
#pragma unroll
    for (int sub = 0; sub < KT; ++sub) {
        if (sub >= n_sub) continue;
        __syncthreads();                                     // K stages / previous staged tile are consumed
        {
            const int row = wave * 32 + n;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float4 v = make_float4(acc[sub][kb][4 * g], acc[sub][kb][4 * g + 1],
                                           acc[sub][kb][4 * g + 2], acc[sub][kb][4 * g + 3]);
                    *reinterpret_cast<float4*>(outs + row * OUT_LD + 32 * kb + 8 * g + 4 * hh) = v;
                }
        }
        __syncthreads();
        // a tile that lies inside the map and below the causal limit for all its rows takes the
        // branch-free path: all 8 loads of a thread are in flight before the first is used
        const long long k_first = (long long)key0 + sub * 64;
        bool interior = vec_ok && qb * BM + BM <= a.Lq && k_first + 63 <= (long long)a.Lk - 1;
        if (a.causal) interior = interior && k_first + 63 <= (long long)qb * BM + off;
        if (interior) {
            float* base = a.abar + ((size_t)h * a.Lq + (size_t)qb * BM + (tid >> 4)) * a.Lk + k_first + c4;
            float4 o[8];
#pragma unroll
            for (int pass = 0; pass < 8; ++pass)
                o[pass] = *reinterpret_cast<const float4*>(base + (size_t)pass * (4 * NW) * a.Lk);
#pragma unroll
            for (int pass = 0; pass < 8; ++pass) {
                const float4 v = *reinterpret_cast<const float4*>(outs + (pass * (4 * NW) + (tid >> 4)) * OUT_LD + c4);
                o[pass].x = fmaf(a.weight, v.x, o[pass].x);
                o[pass].y = fmaf(a.weight, v.y, o[pass].y);
                o[pass].z = fmaf(a.weight, v.z, o[pass].z);
                o[pass].w = fmaf(a.weight, v.w, o[pass].w);
            }
#pragma unroll
            for (int pass = 0; pass < 8; ++pass)
                *reinterpret_cast<float4*>(base + (size_t)pass * (4 * NW) * a.Lk) = o[pass];
            continue;
        }
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int r = pass * (4 * NW) + (tid >> 4);
            const int q = qb * BM + r;
            if (q >= a.Lq) continue;
            long long last_key = (long long)a.Lk - 1;        // last key of this row that is accumulated
            if (a.causal) last_key = min(last_key, (long long)q + off);
            const long long k = k_first + c4;
            if (k > last_key) continue;
            const float4 v = *reinterpret_cast<const float4*>(outs + r * OUT_LD + c4);
            float* dst = a.abar + ((size_t)h * a.Lq + q) * a.Lk + k;
            if (vec_ok && k + 3 <= last_key) {
                float4 o = *reinterpret_cast<float4*>(dst);
                o.x = fmaf(a.weight, v.x, o.x);
                o.y = fmaf(a.weight, v.y, o.y);
                o.z = fmaf(a.weight, v.z, o.z);
                o.w = fmaf(a.weight, v.w, o.w);
                *reinterpret_cast<float4*>(dst) = o;
            } else {
                const float ve[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k + e <= last_key) dst[e] = fmaf(a.weight, ve[e], dst[e]);
            }
        }
    }
}

// lse2 = lse * log2(e): the row statistics as the attention forward call returns them (natural
// logarithm), in the form the accumulation kernel reads.
__global__ __launch_bounds__(256) void lse_to_base2_kernel(const float* __restrict__ lse, float* __restrict__ lse2,
                                                            long long n)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) lse2[i] = lse[i] * kLog2e;                    // -inf (a query without keys) stays -inf
}

template <int D>
hipError_t launch_d(const MapArgs& a, const float* lse, hipStream_t stream)
{
    constexpr int NW = 4, KT = 2;
    const int nQB = (a.Lq + 32 * NW - 1) / (32 * NW), nKG = (a.Lk + 64 * KT - 1) / (64 * KT);
    if (lse) {
        const long long n = (long long)a.B * a.H * a.Lq;
        hipLaunchKernelGGL(lse_to_base2_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, lse,
                           a.lse2, n);
    } else {
        hipLaunchKernelGGL((row_lse_kernel<D, NW>), dim3((unsigned)(a.B * a.H * nQB)), dim3(64 * NW), 0,
                           stream, a, nQB);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((map_accumulate_kernel<D, NW, KT>), dim3((unsigned)(a.H * nQB * nKG)),
                       dim3(64 * NW), 0, stream, a, nQB, nKG);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention_maps(const MapArgs& a, const float* lse, hipStream_t stream)
{
    switch (a.D) {
        case 32: return launch_d<32>(a, lse, stream);
        case 64: return launch_d<64>(a, lse, stream);
        case 128: return launch_d<128>(a, lse, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ap
