// Masked attention forward on the bf16 matrix cores (Section 3.2, masked-attention equation).
//
// One workgroup per block row of the layout (block_m = 32 * NW queries, one wavefront per 32
// queries).  The workgroup walks only the stored tiles of its block row.  Per tile:
//   1. the 64 key rows and 64 value rows are staged in LDS with coalesced 128-bit loads;
//   2. S^T = K Q^T on v_mfma_f32_32x32x16_bf16, so that every lane holds scores of ONE query
//      (lane % 32) for 32 of the 64 keys -- the row maximum is an in-register reduction plus
//      a single exchange with lane ^ 32, and the row sum needs no exchange until the end;
//   3. the lane's 64-bit bitmap word (and the causal limit) turns pruned scores into -inf in
//      registers, before the exponential;
//   4. online softmax in fp32 (exp2 with scale*log2(e) folded into one fma);
//   5. O^T += V^T P^T on the matrix cores: the S^T accumulator registers already have the
//      lane layout of the P^T operand, and V^T is read from the row-major LDS tile with the
//      transposing LDS read, so nothing is shuffled.
// O is normalised and written once at the end together with the optional log-sum-exp.
//
// Matrix-core register layouts used below (32x32x16, 64 lanes, l = lane):
//   A[m][k]: m = l % 32, k = 8*(l/32) + e, e = 0..7        B[k][n]: n = l % 32, same k
//   C[m][n]: n = l % 32, m = 8*(i/4) + 4*(l/32) + i%4, i = 0..15
// The contraction index of the second product runs over keys in the order the S^T registers
// hold them (slot (l/32, e) of 16-key step ks is key 16*ks + 8*(e/4) + 4*(l/32) + e%4); both
// operands use the same order, which leaves the sum unchanged.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr int kBN = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int D>
struct Tile {
    static constexpr int KSTR = D + 8;                       // bf16 elements per LDS key row
    static constexpr int VSTR = (D == 32) ? 96 : D + 32;     // bf16 elements per LDS value row
};

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void fwd_mfma_kernel(FwdArgs a, int nQB)
{
    constexpr int BM = 32 * NW;
    constexpr int NT = 64 * NW;
    constexpr int KSTR = Tile<D>::KSTR;
    constexpr int VSTR = Tile<D>::VSTR;
    constexpr int KSTEPS = D / 16;                           // contraction steps of Q K^T
    constexpr int DBLK = D / 32;                             // 32-wide blocks of the head dim
    constexpr int CPR = D / 8;                               // 16-byte chunks per row
    constexpr int CHUNKS = (kBN * CPR) / NT;                 // chunks per thread per operand
    static_assert((kBN * CPR) % NT == 0, "tile must divide evenly over the threads");

    __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * KSTR];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[kBN * VSTR];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int n = lane & 31;                                 // query inside the wavefront's 32
    const int hh = lane >> 5;                                // which half of the key slots

    // block row: long causal rows are issued first
    const int bid = blockIdx.x;
    const int qb = nQB - 1 - (bid % nQB);
    const int h = (bid / nQB) % a.H;
    const int b = bid / (nQB * a.H);

    const uint16_t* Qp = (const uint16_t*)a.Q + (size_t)b * a.sq[0] + (size_t)h * a.sq[1];
    const uint16_t* Kp = (const uint16_t*)a.K + (size_t)b * a.sk[0] + (size_t)h * a.sk[1];
    const uint16_t* Vp = (const uint16_t*)a.V + (size_t)b * a.sv[0] + (size_t)h * a.sv[1];
    uint16_t* Op = (uint16_t*)a.O + (size_t)b * a.so[0] + (size_t)h * a.so[1];

    const int brow = wave * 32 + n;                          // row inside the block row
    const int qrow = qb * BM + brow;                         // this lane's query
    const bool row_ok = qrow < a.Lq;

    // Q^T operand, resident in registers for the whole kernel
    bf16x8 qreg[KSTEPS];
    {
        const uint16_t* qr = Qp + (size_t)(row_ok ? qrow : a.Lq - 1) * a.sq[2] + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            qreg[kk] = *reinterpret_cast<const bf16x8*>(qr + 16 * kk);
    }

    f32x16 oacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m = -INFINITY;                                     // running max of raw scores
    float lsum = 0.f;                                        // this lane's share of the row sum
    const float sc = a.scale * kLog2e;

    const int r = h * nQB + qb;
    const int t_begin = a.row_ptr[r], t_end = a.row_ptr[r + 1];
    const long long off = (long long)a.Lk - a.Lq;
    const long long diag = (long long)qrow + off;            // last visible key if causal
    const long long block_diag = (long long)qb * BM + (BM - 1) + off;

    for (int t = t_begin; t < t_end; ++t) {
        const int k0 = a.col_idx[t] * kBN;
        if (a.causal && (long long)k0 > block_diag) break;   // this and all later tiles are hidden

        uint64_t word = a.bitmaps[(size_t)t * BM + brow];
        if (a.causal) {
            const long long lim = diag - k0;
            if (lim < 0) word = 0;
            else if (lim < 63) word &= (2ull << lim) - 1ull;
        }

        __syncthreads();                                     // everyone is done with the previous tile
        {
            uint4 kbuf[CHUNKS], vbuf[CHUNKS];
#pragma unroll
            for (int u = 0; u < CHUNKS; ++u) {
                const int c = tid + u * NT;
                const int rr = c / CPR, e0 = (c % CPR) * 8;
                int row = k0 + rr;
                row = row < a.Lk ? row : a.Lk - 1;
                kbuf[u] = *reinterpret_cast<const uint4*>(Kp + (size_t)row * a.sk[2] + e0);
                vbuf[u] = *reinterpret_cast<const uint4*>(Vp + (size_t)row * a.sv[2] + e0);
            }
#pragma unroll
            for (int u = 0; u < CHUNKS; ++u) {
                const int c = tid + u * NT;
                const int rr = c / CPR, e0 = (c % CPR) * 8;
                *reinterpret_cast<uint4*>(Ks + rr * KSTR + e0) = kbuf[u];
                *reinterpret_cast<uint4*>(Vs + rr * VSTR + e0) = vbuf[u];
            }
        }
        __syncthreads();

        if (__ballot(word != 0) == 0) continue;              // nothing visible for these 32 queries

        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 kreg = *reinterpret_cast<const bf16x8*>(
                    Ks + (kb * 32 + n) * KSTR + 16 * kk + 8 * hh);
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg, qreg[kk], sacc[kb], 0, 0, 0);
            }
        }

        // ---- mask in registers, row maximum
        const uint64_t wsh = word >> (4 * hh);
        const uint32_t wbits[2] = {(uint32_t)wsh, (uint32_t)(wsh >> 32)};
        float tmax = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int pos = 8 * (i / 4) + (i % 4);
                const float s = ((wbits[kb] >> pos) & 1u) ? sacc[kb][i] : -INFINITY;
                sacc[kb][i] = s;
                tmax = fmaxf(tmax, s);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));

        // ---- online softmax
        const float m_new = fmaxf(m, tmax);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m - m_use) * sc);
        const float msc = m_use * sc;
        m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], sc, -msc));
                sacc[kb][i] = p;
                psum += p;
            }
        lsum = lsum * alpha + psum;
        if (__ballot(alpha != 1.0f) != 0) {
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 pb;
#pragma unroll
            for (int e = 0; e < 8; ++e) pb[e] = (__bf16)sacc[ks >> 1][8 * (ks & 1) + e];
            const int i16 = lane & 15, g = (lane >> 4) & 1;
            const int vrow = 16 * ks + 4 * hh + (i16 >> 2);
            const int vcol = 16 * g + 4 * (i16 & 3);
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                lds_bf16x4* p0 = (lds_bf16x4*)((__attribute__((address_space(3))) uint16_t*)Vs +
                                               vrow * VSTR + 32 * db + vcol);
                lds_bf16x4* p1 = (lds_bf16x4*)((__attribute__((address_space(3))) uint16_t*)Vs +
                                               (vrow + 8) * VSTR + 32 * db + vcol);
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(p0);
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(p1);
                const bf16x8 vreg = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vreg, pb, oacc[db], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: normalise, write O (bf16, round to nearest even) and lse
    const float ltot = lsum + __shfl_xor(lsum, 32, 64);
    if (!row_ok) return;
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    uint16_t* orow = Op + (size_t)qrow * a.so[2];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            uint2 w;
            w.x = pack_bf16_rne(oacc[db][4 * g4] * inv, oacc[db][4 * g4 + 1] * inv);
            w.y = pack_bf16_rne(oacc[db][4 * g4 + 2] * inv, oacc[db][4 * g4 + 3] * inv);
            *reinterpret_cast<uint2*>(orow + 32 * db + 8 * g4 + 4 * hh) = w;
        }
    if (a.lse && hh == 0)
        a.lse[((size_t)b * a.H + h) * a.Lq + qrow] =
            ltot > 0.f ? (m * sc + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
}

template <int D, int NW>
hipError_t launch_one(const FwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + 32 * NW - 1) / (32 * NW);
    const long long blocks = (long long)nQB * a.H * a.B;
    hipLaunchKernelGGL((fwd_mfma_kernel<D, NW>), dim3((unsigned)blocks), dim3(64 * NW), 0, stream, a, nQB);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_mfma(const FwdArgs& a, hipStream_t stream)
{
    const bool wide = a.block_m == 128;
    switch (a.D) {
    case 32: return wide ? launch_one<32, 4>(a, stream) : launch_one<32, 2>(a, stream);
    case 64: return wide ? launch_one<64, 4>(a, stream) : launch_one<64, 2>(a, stream);
    case 128: return wide ? launch_one<128, 4>(a, stream) : launch_one<128, 2>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ap
