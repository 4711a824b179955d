// Layer-wise percentile threshold and pruning mask (Section 3.2, paragraph before Eq. (2), and
// Eq. (2)).
//
// tau is the order statistic of rank floor(p * N) among the N participating entries of the mean
// maps of all heads of a layer.  It is found exactly by a radix selection over the entries' bit
// patterns, most significant digit first (12 + 10 + 10 bits): each pass histograms one digit of
// the entries that agree with the digits fixed so far, and a one-workgroup kernel picks the bin
// that holds the wanted rank.  A last pass compares every entry with tau.  All passes stream
// the maps once; the kernels are bound by HBM reads (4 bytes per entry and pass).
//
// Float bit patterns are mapped to unsigned keys whose integer order is the numeric order
// (sign bit flipped for non-negative values, all bits flipped for negative ones; -0 counts as +0).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

constexpr int kMaxBins = 4096;

struct SelectState {
    unsigned long long hist[kMaxBins];
    unsigned long long rank;     // wanted rank among the entries that match `prefix`
    uint32_t prefix;             // key digits fixed so far (lower digits zero)
    uint32_t pad;
};

__device__ __forceinline__ uint32_t key_of(float v)
{
    uint32_t b = __float_as_uint(v);
    if ((b << 1) == 0) b = 0;                                // -0 -> +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float value_of(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

__global__ void select_init_kernel(SelectState* st, unsigned long long rank, float* tau_out, int none)
{
    for (int i = threadIdx.x; i < kMaxBins; i += blockDim.x) st->hist[i] = 0;
    if (threadIdx.x == 0) {
        st->rank = rank;
        st->prefix = 0;
        if (none && tau_out) *tau_out = INFINITY;            // rank N: everything is pruned
    }
}

// Rows of the maps are dealt to workgroups in contiguous chunks; inside a workgroup `tpr`
// threads (a power of two) share a row and 256 / tpr rows are in flight, so short rows still
// fill the wavefronts.  Only the visible prefix of a row is read.
struct RowWalk {
    const float* abar;
    long long rows;              // H * Lq
    int Lq, Lk;
    int causal;
    int tpr;
};

template <typename F>
__device__ __forceinline__ void for_each_visible(const RowWalk& w, F&& f)
{
    const long long chunk = (w.rows + gridDim.x - 1) / gridDim.x;
    const long long r0 = (long long)blockIdx.x * chunk;
    const long long r1 = min(w.rows, r0 + chunk);
    const int rpi = 256 / w.tpr;
    const int tr = threadIdx.x / w.tpr, tc = threadIdx.x % w.tpr;
    const bool vec_ok = (w.Lk & 3) == 0;
    const long long off = (long long)w.Lk - w.Lq;
    for (long long r = r0 + tr; r < r1; r += rpi) {
        int nvis = w.Lk;
        if (w.causal) nvis = (int)min((long long)w.Lk, (long long)(r % w.Lq) + off + 1);
        const float* src = w.abar + (size_t)r * w.Lk;
        for (int j = tc * 4; j < nvis; j += w.tpr * 4) {
            if (vec_ok && j + 3 < nvis) {
                const float4 v = *reinterpret_cast<const float4*>(src + j);
                f(v.x); f(v.y); f(v.z); f(v.w);
            } else {
                for (int e = 0; e < 4 && j + e < nvis; ++e) f(src[j + e]);
            }
        }
    }
}

template <int SHIFT, int BITS>
__global__ __launch_bounds__(256) void radix_hist_kernel(RowWalk w, SelectState* st)
{
    constexpr int NB = 1 << BITS;
    constexpr uint32_t HIGH = (SHIFT + BITS >= 32) ? 0u : ~((1u << (SHIFT + BITS)) - 1u);
    __shared__ uint32_t h[NB];
    for (int i = threadIdx.x; i < NB; i += 256) h[i] = 0;
    __syncthreads();
    const uint32_t prefix = st->prefix;
    for_each_visible(w, [&](float v) {
        const uint32_t key = key_of(v);
        if ((key & HIGH) == prefix) atomicAdd(&h[(key >> SHIFT) & (NB - 1)], 1u);
    });
    __syncthreads();
    for (int i = threadIdx.x; i < NB; i += 256)
        if (h[i]) atomicAdd(&st->hist[i], (unsigned long long)h[i]);
}

// One workgroup: find the bin whose cumulative count passes the wanted rank, fix that digit,
// and clear the histogram for the next pass.
template <int SHIFT, int BITS, bool LAST>
__global__ __launch_bounds__(256) void radix_select_kernel(SelectState* st, float* tau_out)
{
    constexpr int NB = 1 << BITS;
    constexpr int PER = NB / 256;
    __shared__ unsigned long long part[256];
    const int t = threadIdx.x;
    const unsigned long long rank = st->rank;
    unsigned long long mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) mine += st->hist[t * PER + i];
    part[t] = mine;
    __syncthreads();
    unsigned long long before = 0;
    for (int i = 0; i < t; ++i) before += part[i];
    __syncthreads();                                         // everybody has read st->rank and part[]
    if (rank >= before && rank < before + mine) {            // exactly one thread
        unsigned long long cum = before;
        for (int i = 0; i < PER; ++i) {
            const unsigned long long c = st->hist[t * PER + i];
            if (rank < cum + c) {
                const uint32_t prefix = st->prefix | ((uint32_t)(t * PER + i) << SHIFT);
                st->prefix = prefix;
                st->rank = rank - cum;
                if (LAST && tau_out) *tau_out = value_of(prefix);
                break;
            }
            cum += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER; ++i) st->hist[t * PER + i] = 0;
}

__global__ __launch_bounds__(256) void prune_mask_kernel(RowWalk w, const SelectState* st,
                                                         uint8_t* mask, int none)
{
    const uint32_t tau_key = st->prefix;
    const long long chunk = (w.rows + gridDim.x - 1) / gridDim.x;
    const long long r0 = (long long)blockIdx.x * chunk;
    const long long r1 = min(w.rows, r0 + chunk);
    const int rpi = 256 / w.tpr;
    const int tr = threadIdx.x / w.tpr, tc = threadIdx.x % w.tpr;
    const bool vec_ok = (w.Lk & 3) == 0;
    const long long off = (long long)w.Lk - w.Lq;
    for (long long r = r0 + tr; r < r1; r += rpi) {
        int nvis = w.Lk;
        if (w.causal) nvis = (int)min((long long)w.Lk, (long long)(r % w.Lq) + off + 1);
        if (none) nvis = 0;
        const float* src = w.abar + (size_t)r * w.Lk;
        uint8_t* dst = mask + (size_t)r * w.Lk;
        for (int j = tc * 4; j < w.Lk; j += w.tpr * 4) {
            if (vec_ok) {                                    // 4 entries, 4 output bytes
                uint32_t out = 0;
                if (j + 3 < nvis) {
                    const float4 v = *reinterpret_cast<const float4*>(src + j);
                    out = (key_of(v.x) >= tau_key ? 1u : 0u) | (key_of(v.y) >= tau_key ? 0x100u : 0u) |
                          (key_of(v.z) >= tau_key ? 0x10000u : 0u) | (key_of(v.w) >= tau_key ? 0x1000000u : 0u);
                } else {
                    for (int e = 0; e < 4 && j + e < nvis; ++e)
                        if (key_of(src[j + e]) >= tau_key) out |= 1u << (8 * e);
                }
                *reinterpret_cast<uint32_t*>(dst + j) = out;
            } else {
                for (int e = 0; e < 4 && j + e < w.Lk; ++e)
                    dst[j + e] = (j + e < nvis && key_of(src[j + e]) >= tau_key) ? 1 : 0;
            }
        }
    }
}

}  // namespace

size_t prune_mask_workspace_bytes() { return sizeof(SelectState); }

hipError_t launch_prune_mask(const float* abar, int H, int Lq, int Lk, int causal,
                             unsigned long long rank, bool none, uint8_t* mask, float* tau_out,
                             void* workspace, hipStream_t stream)
{
    SelectState* st = reinterpret_cast<SelectState*>(workspace);
    RowWalk w;
    w.abar = abar;
    w.rows = (long long)H * Lq;
    w.Lq = Lq;
    w.Lk = Lk;
    w.causal = causal;
    int tpr = 1;                                             // threads per row: each takes 4 entries a step
    while (tpr < 256 && tpr * 4 < Lk) tpr <<= 1;
    w.tpr = tpr;
    // enough workgroups to fill the chip several times over, but no fewer than 256/tpr rows each
    const long long rows_per_step = 256 / tpr;
    long long grid = (w.rows + rows_per_step - 1) / rows_per_step;
    if (grid > 4096) grid = 4096;

    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(256), 0, stream, st, rank, tau_out, none ? 1 : 0);
    if (!none) {
        hipLaunchKernelGGL((radix_hist_kernel<20, 12>), dim3((unsigned)grid), dim3(256), 0, stream, w, st);
        hipLaunchKernelGGL((radix_select_kernel<20, 12, false>), dim3(1), dim3(256), 0, stream, st, tau_out);
        hipLaunchKernelGGL((radix_hist_kernel<10, 10>), dim3((unsigned)grid), dim3(256), 0, stream, w, st);
        hipLaunchKernelGGL((radix_select_kernel<10, 10, false>), dim3(1), dim3(256), 0, stream, st, tau_out);
        hipLaunchKernelGGL((radix_hist_kernel<0, 10>), dim3((unsigned)grid), dim3(256), 0, stream, w, st);
        hipLaunchKernelGGL((radix_select_kernel<0, 10, true>), dim3(1), dim3(256), 0, stream, st, tau_out);
    }
    hipLaunchKernelGGL(prune_mask_kernel, dim3((unsigned)grid), dim3(256), 0, stream, w, st, mask, none ? 1 : 0);
    return hipGetLastError();
}

}  // namespace ap
