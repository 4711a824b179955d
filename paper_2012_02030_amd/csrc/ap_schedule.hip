// Visit schedule: a derived, deterministic re-packing of the block-sparse layout.
//
// A mask that keeps a band next to the diagonal (the constant context window in the figure of
// Section 5.1) plus scattered isolated connections has a kept entry in almost every 64x64 tile
// of a long causal sequence, so walking "every non-empty tile" would cost as much as dense
// attention.  The schedule keeps tiles with many distinct visible key columns as they are
// (64 consecutive keys) and packs the visible columns of all other tiles of a block row,
// in ascending order, into gathered tiles of 64 arbitrary keys with their own bitmaps.  The
// causal limit is folded into the bitmaps here, so the attention kernel applies bitmaps only.
//
// One workgroup per block row, one thread per query row.  All control flow depends only on the
// OR of the row words (workgroup-uniform), so the emitted order is fixed: no atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

// OR over all threads of the workgroup (blockDim.x = 64 or 128); every thread gets the result.
__device__ __forceinline__ uint64_t block_or(uint64_t v, uint64_t* red)
{
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        lo |= __shfl_xor(lo, off, 64);
        hi |= __shfl_xor(hi, off, 64);
    }
    uint64_t w = ((uint64_t)hi << 32) | lo;
    if (blockDim.x > 64) {
        __syncthreads();                                   // previous use of red[] is over
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
        __syncthreads();
        w = red[0] | red[1];
    }
    return w;
}

__global__ __launch_bounds__(128) void build_schedule_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const uint64_t* __restrict__ bitmaps, int nQB, int Lq, int Lk, int BM, long long cap,
    int causal, int min_cols, Schedule s)
{
    __shared__ uint64_t red[2];
    const int r = blockIdx.x;
    const int qb = r % nQB;
    const int row = threadIdx.x;                           // 0 .. BM-1
    const long long diag = (long long)qb * BM + row + ((long long)Lk - Lq);

    const int t0 = row_ptr[r];
    const int t1 = (int)min((long long)row_ptr[r + 1], cap);   // a truncated layout is never read past cap
    int n_out = 0;                                         // entry slots handed out so far
    uint64_t tail_word = 0;                                // this row's bits of the open gathered entry
    int fill = 0;                                          // columns in the open gathered entry
    size_t tail_slot = 0;                                  // its slot, reserved when its first column arrives

    // Two passes over the stored tiles: first the entries that stay runs of 64 consecutive keys,
    // then the gathered ones, so that the attention kernel meets a gathered entry (whose keys it
    // must fetch before it can load anything) only after it has other loads in flight.
    for (int pass = 0; pass < 2; ++pass) {
        for (int t = t0; t < t1; ++t) {
            const int k0 = col_idx[t] * 64;
            uint64_t word = bitmaps[(size_t)t * BM + row];
            if (causal) {
                const long long lim = diag - k0;
                if (lim < 0) word = 0;
                else if (lim < 63) word &= (2ull << lim) - 1ull;
            }
            uint64_t colmask = block_or(word, red);
            const int ncols = __popcll(colmask);
            if (ncols == 0) continue;                      // nothing visible
            const bool consecutive = ncols >= min_cols;
            if (consecutive != (pass == 0)) continue;
            if (consecutive) {                             // keep as a tile of 64 consecutive keys
                const size_t e = (size_t)t0 + n_out;
                if (row == 0) s.start[e] = k0;
                s.bitmaps[e * BM + row] = word;
                ++n_out;
                continue;
            }
            while (colmask) {                              // append the visible columns, ascending
                const int bit = __ffsll((long long)colmask) - 1;
                colmask &= colmask - 1;
                if (fill == 0) {                           // open a gathered entry: one per <= 64 columns,
                    tail_slot = (size_t)t0 + n_out;        // so never more entries than visible tiles
                    ++n_out;
                    if (row == 0) s.start[tail_slot] = -1;
                }
                tail_word |= ((word >> bit) & 1ull) << fill;
                if (row == 0) s.cols[tail_slot * 64 + fill] = k0 + bit;
                if (++fill == 64) {
                    s.bitmaps[tail_slot * BM + row] = tail_word;
                    tail_word = 0;
                    fill = 0;
                }
            }
        }
    }
    if (fill > 0) {                                        // last, partly filled gathered entry
        for (int c = fill + row; c < 64; c += BM) s.cols[tail_slot * 64 + c] = Lk;   // empty slot: reads as zeros
        s.bitmaps[tail_slot * BM + row] = tail_word;
    }
    if (row == 0) s.cnt[r] = n_out;
}

}  // namespace

hipError_t launch_build_schedule(const int32_t* row_ptr, const int32_t* col_idx,
                                 const uint64_t* bitmaps, int H, int Lq, int Lk, int BM,
                                 long long cap, int causal, int min_cols, const Schedule& s,
                                 hipStream_t stream)
{
    const int nQB = (Lq + BM - 1) / BM;
    hipLaunchKernelGGL(build_schedule_kernel, dim3((unsigned)(H * nQB)), dim3(BM), 0, stream, row_ptr,
                       col_idx, bitmaps, nQB, Lq, Lk, BM, cap, causal, min_cols, s);
    return hipGetLastError();
}

}  // namespace ap
