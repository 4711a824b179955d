// Masked attention forward in fp32 vector arithmetic (Section 3.2, masked-attention equation).
//
// One workgroup of four wavefronts per 64-query block row; in every wavefront each lane owns one
// query, and wavefront w takes the key columns c with c % 4 == w of every tile (interleaved, so a
// diagonal tile's visible columns spread evenly).  The workgroup walks the stored tiles of its block
// row, stages the tile's 64 key rows and 64 value rows in LDS (coalesced 128-bit loads), and every
// wavefront, for each of its key columns that any lane keeps, forms the scaled dot product (LDS
// broadcast reads), masks it with the lane's bitmap bit, and folds it into an online softmax of its
// own.  The four partial states (maximum, sum, accumulator) are merged through LDS at the end.
// This is the fp32 path (and a matrix-core-free cross-check for bf16 storage).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

constexpr int kBM = 64;
constexpr int kBN = 64;
constexpr int kNW = 4;                                 // wavefronts per block row
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even fp32 -> bf16 bits (inputs are finite or inf, never NaN here)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Load 64 rows x D elements of X (rows row0.., clamped to n_rows-1) into LDS as fp32.
template <bool BF16, int D>
__device__ __forceinline__ void stage_rows(float* __restrict__ dst, const void* __restrict__ base,
                                           long long stride_seq, int row0, int n_rows, int tid)
{
    constexpr int EPC = BF16 ? 8 : 4;                  // elements per 16-byte chunk
    constexpr int CPR = D / EPC;                       // chunks per row
    constexpr int LSTR = D + 4;                        // LDS row stride in floats
    for (int c = tid; c < kBN * CPR; c += 64 * kNW) {
        const int r = c / CPR;
        const int e0 = (c % CPR) * EPC;
        int row = row0 + r;
        row = row < n_rows ? row : n_rows - 1;
        float* d = dst + r * LSTR + e0;
        if (BF16) {
            const uint4 v = *reinterpret_cast<const uint4*>(
                reinterpret_cast<const uint16_t*>(base) + (size_t)row * stride_seq + e0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                d[2 * k] = bf16_bits_to_float(w[k] & 0xffffu);
                d[2 * k + 1] = bf16_bits_to_float(w[k] >> 16);
            }
        } else {
            const float4 v = *reinterpret_cast<const float4*>(
                reinterpret_cast<const float*>(base) + (size_t)row * stride_seq + e0);
            *reinterpret_cast<float4*>(d) = v;
        }
    }
}

template <bool BF16, int D>
__global__ __launch_bounds__(64 * kNW) void fwd_valu_kernel(const int32_t* __restrict__ p_row_ptr, int nQB, FwdArgs a)
{
    constexpr int LSTR = D + 4;
    constexpr int STAGE = 2 * kBN * LSTR + kBN * 64;   // floats: key rows, value rows, scores
    constexpr int MERGE = 2 * (D + 2) * 64;            // two partial states, [state][field][lane]
    static_assert(MERGE <= STAGE, "the merge buffers reuse the staging area");
    __shared__ __attribute__((aligned(16))) float smem[STAGE];
    float* Ks = smem;
    float* Vs = Ks + kBN * LSTR;
    float* Ss = Vs + kBN * LSTR;                       // [key column][lane]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qb = nQB - 1 - (int)blockIdx.x;          // long causal rows first
    const int h = blockIdx.y;
    const int b = blockIdx.z;
    // the row pointers travel as a leading argument (preloaded into registers at wavefront start),
    // so this load does not wait for the argument block
    const int r = h * nQB + qb;
    const int t_begin = p_row_ptr[r], t_end = p_row_ptr[r + 1];
    const int i = qb * kBM + lane;                     // this lane's query
    const bool row_ok = i < a.Lq;
    const int iq = row_ok ? i : a.Lq - 1;

    const size_t esz = BF16 ? 2 : 4;
    const char* Qp = (const char*)a.Q + ((size_t)b * a.sq[0] + (size_t)h * a.sq[1]) * esz;
    const char* Kp = (const char*)a.K + ((size_t)b * a.sk[0] + (size_t)h * a.sk[1]) * esz;
    const char* Vp = (const char*)a.V + ((size_t)b * a.sv[0] + (size_t)h * a.sv[1]) * esz;
    char* Op = (char*)a.O + ((size_t)b * a.so[0] + (size_t)h * a.so[1]) * esz;

    // query row, pre-multiplied by scale*log2(e): scores live in the log2 domain
    const float qs = a.scale * kLog2e;
    float q[D];
    if (BF16) {
        const uint16_t* qr = (const uint16_t*)Qp + (size_t)iq * a.sq[2];
#pragma unroll
        for (int t = 0; t < D; t += 8) {
            const uint4 v = *reinterpret_cast<const uint4*>(qr + t);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                q[t + 2 * k] = bf16_bits_to_float(w[k] & 0xffffu) * qs;
                q[t + 2 * k + 1] = bf16_bits_to_float(w[k] >> 16) * qs;
            }
        }
    } else {
        const float* qr = (const float*)Qp + (size_t)iq * a.sq[2];
#pragma unroll
        for (int t = 0; t < D; t += 4) {
            const float4 v = *reinterpret_cast<const float4*>(qr + t);
            q[t] = v.x * qs; q[t + 1] = v.y * qs; q[t + 2] = v.z * qs; q[t + 3] = v.w * qs;
        }
    }

    float acc[D];
#pragma unroll
    for (int t = 0; t < D; ++t) acc[t] = 0.f;
    float m = -INFINITY;                               // running max (log2 domain)
    float l = 0.f;                                     // running sum of 2^(s - m)

    const long long diag = (long long)i + (a.Lk - a.Lq);   // last visible key if causal

    for (int t = t_begin; t < t_end; ++t) {
        const int kb = a.col_idx[t];
        const int k0 = kb * kBN;
        uint64_t word = row_ok ? a.bitmaps[(size_t)t * kBM + lane] : 0ull;
        if (a.causal) {
            const long long lim = diag - k0;           // last visible column inside the tile
            if (lim < 0) word = 0;
            else if (lim < 63) word &= (2ull << lim) - 1ull;
        }
        // every wavefront holds the same 64 queries: the same decision in all four
        if (__ballot(word != 0) == 0) continue;        // nothing visible in this tile

        __syncthreads();                               // previous tile's LDS reads are done
        stage_rows<BF16, D>(Ks, Kp, a.sk[2], k0, a.Lk, tid);
        stage_rows<BF16, D>(Vs, Vp, a.sv[2], k0, a.Lk, tid);
        __syncthreads();

        // scores of this wavefront's columns; pruned entries stay at -inf
        float tile_max = -INFINITY;
        unsigned long long used = 0;                   // columns some lane keeps (wave-uniform)
        for (int c = wave; c < kBN; c += kNW) {
            const bool mine = (word >> c) & 1ull;
            if (__ballot(mine) == 0) continue;
            used |= 1ull << c;
            const float* kr = Ks + c * LSTR;
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int e = 0; e < D; e += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(kr + e);
                s0 = fmaf(q[e], kv.x, s0);
                s1 = fmaf(q[e + 1], kv.y, s1);
                s2 = fmaf(q[e + 2], kv.z, s2);
                s3 = fmaf(q[e + 3], kv.w, s3);
            }
            const float s = mine ? (s0 + s1) + (s2 + s3) : -INFINITY;
            Ss[c * 64 + lane] = s;
            tile_max = fmaxf(tile_max, s);
        }

        // online softmax update
        const float m_new = fmaxf(m, tile_max);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);   // m = -inf -> 0
        l *= alpha;
#pragma unroll
        for (int e = 0; e < D; ++e) acc[e] *= alpha;
        m = m_new;

        unsigned long long rest = used;
        while (rest) {
            const int c = __ffsll((long long)rest) - 1;
            rest &= rest - 1;
            const float p = __builtin_amdgcn_exp2f(Ss[c * 64 + lane] - m_use);   // -inf -> 0
            l += p;
            const float* vr = Vs + c * LSTR;
#pragma unroll
            for (int e = 0; e < D; e += 4) {
                const float4 vv = *reinterpret_cast<const float4*>(vr + e);
                acc[e] = fmaf(p, vv.x, acc[e]);
                acc[e + 1] = fmaf(p, vv.y, acc[e + 1]);
                acc[e + 2] = fmaf(p, vv.z, acc[e + 2]);
                acc[e + 3] = fmaf(p, vv.w, acc[e + 3]);
            }
        }
    }

    // merge the four partial states pairwise through LDS: (1 -> 0, 3 -> 2), then 2 -> 0
    auto put = [&](int slot) {
        float* p = smem + slot * (D + 2) * 64 + lane;
        p[0] = m;
        p[64] = l;
#pragma unroll
        for (int e = 0; e < D; ++e) p[(2 + e) * 64] = acc[e];
    };
    auto take = [&](int slot) {
        const float* p = smem + slot * (D + 2) * 64 + lane;
        const float m2 = p[0], l2 = p[64];
        const float m_new = fmaxf(m, m2);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float a1 = __builtin_amdgcn_exp2f(m - m_use), a2 = __builtin_amdgcn_exp2f(m2 - m_use);
        l = l * a1 + l2 * a2;
#pragma unroll
        for (int e = 0; e < D; ++e) acc[e] = acc[e] * a1 + p[(2 + e) * 64] * a2;
        m = m_new;
    };
    __syncthreads();                                   // the staging area is free
    if (wave & 1) put(wave >> 1);
    __syncthreads();
    if (!(wave & 1)) take(wave >> 1);
    __syncthreads();
    if (wave == 2) put(0);
    __syncthreads();
    if (wave != 0 || !row_ok) return;
    take(0);

    const float inv = l > 0.f ? 1.f / l : 0.f;
    if (BF16) {
        uint16_t* orow = (uint16_t*)Op + (size_t)i * a.so[2];
#pragma unroll
        for (int e = 0; e < D; e += 8) {
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                w[k] = float_to_bf16_bits(acc[e + 2 * k] * inv) |
                       (float_to_bf16_bits(acc[e + 2 * k + 1] * inv) << 16);
            *reinterpret_cast<uint4*>(orow + e) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    } else {
        float* orow = (float*)Op + (size_t)i * a.so[2];
#pragma unroll
        for (int e = 0; e < D; e += 4)
            *reinterpret_cast<float4*>(orow + e) =
                make_float4(acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv);
    }
    if (a.lse)
        a.lse[((size_t)b * a.H + h) * a.Lq + i] =
            l > 0.f ? (m + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
}

template <bool BF16, int D>
hipError_t launch_one(const FwdArgs& a, hipStream_t stream)
{
    const int nQB = (a.Lq + kBM - 1) / kBM;
    hipLaunchKernelGGL((fwd_valu_kernel<BF16, D>), dim3(nQB, a.H, a.B), dim3(64 * kNW), 0, stream, a.row_ptr,
                       nQB, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_valu(const FwdArgs& a, bool bf16, hipStream_t stream)
{
    switch (a.D) {
    case 32: return bf16 ? launch_one<true, 32>(a, stream) : launch_one<false, 32>(a, stream);
    case 64: return bf16 ? launch_one<true, 64>(a, stream) : launch_one<false, 64>(a, stream);
    case 128: return bf16 ? launch_one<true, 128>(a, stream) : launch_one<false, 128>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ap
