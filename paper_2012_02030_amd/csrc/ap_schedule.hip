// Visit schedule: a derived, deterministic re-packing of the block-sparse layout.
//
// A mask that keeps a band next to the diagonal (the constant context window in the figure of
// Section 5.1) plus scattered isolated connections has a kept entry in almost every 64x64 tile
// of a long causal sequence, so walking "every non-empty tile" would cost as much as dense
// attention.  The schedule keeps tiles with many distinct visible key columns as they are
// (64 consecutive keys) and packs the visible columns of all other tiles of a block row into
// gathered tiles of 64 arbitrary keys with their own bitmaps.  The causal limit is folded into
// the bitmaps here, so the attention kernel applies bitmaps only.
//
// The attention kernels give every 32 queries of a block row to one wavefront, and a wavefront
// skips an entry in which its 32 queries keep nothing.  Gathered columns are therefore not packed
// in plain ascending order but grouped by the 32-query groups that use them (first the columns
// used only by group 0, then those whose users span groups 0..1, ..., last those used only by the
// last group; ascending inside a class): an isolated connection is used by one query, so most
// gathered entries then concern one wavefront only and the other one skips them.
//
// One workgroup per block row, one thread per query row.  The bitmap words of up to kSeg tiles are
// brought into LDS with all loads in flight at once, and everything else runs from there.  All
// control flow depends only on OR-reductions of the row words (workgroup-uniform), so the emitted
// order is fixed: no atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

constexpr int kSegWords = 4096;                            // bitmap words held in LDS at a time (32 KB)
constexpr int kSegMax = 64;                                // ... i.e. at most this many tiles (block_m = 64)

// words[t * BM + row], then gm[t * 4 + g]: visible columns of 32-row group g of tile t
__global__ __launch_bounds__(128) void build_schedule_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const uint64_t* __restrict__ bitmaps, int nQB, int Lq, int Lk, int BM, long long cap,
    int causal, int min_cols, Schedule s)
{
    extern __shared__ uint64_t lds64[];
    uint64_t* words = lds64;
    uint64_t* gm = lds64 + kSegWords;
    __shared__ int32_t k0s[kSegMax];
    const int kSeg = kSegWords / BM;                       // tiles per segment

    const int r = blockIdx.x;
    const int qb = r % nQB;
    const int row = threadIdx.x;                           // 0 .. BM-1
    const int NG = BM / 32;                                // 32-row groups (wavefronts of the attention kernel)
    const long long diag = (long long)qb * BM + row + ((long long)Lk - Lq);

    const int t0 = row_ptr[r];
    const int t1 = (int)min((long long)row_ptr[r + 1], cap);   // a truncated layout is never read past cap
    int n_out = 0;                                         // entry slots handed out so far
    uint64_t tail_word = 0;                                // this row's bits of the open gathered entry
    int fill = 0;                                          // columns in the open gathered entry
    size_t tail_slot = 0;                                  // its slot, reserved when its first column arrives

    // Fills LDS with the (causally limited) words of tiles [seg, seg + n) and the visible columns of
    // every 32-row group of each.
    auto load_segment = [&](int seg, int n) {
        __syncthreads();                                   // previous use of the LDS arrays is over
        for (int t = row; t < n; t += BM) k0s[t] = col_idx[seg + t] * 64;
        for (int tb = 0; tb < n; tb += 8) {
            uint64_t w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = tb + u < n ? bitmaps[(size_t)(seg + tb + u) * BM + row] : 0ull;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (tb + u >= n) break;
                uint64_t word = w[u];
                if (causal) {
                    const long long lim = diag - (long long)col_idx[seg + tb + u] * 64;
                    if (lim < 0) word = 0;
                    else if (lim < 63) word &= (2ull << lim) - 1ull;
                }
                words[(size_t)(tb + u) * BM + row] = word;
                uint32_t lo = (uint32_t)word, hi = (uint32_t)(word >> 32);
#pragma unroll
                for (int off = 1; off < 32; off <<= 1) {   // OR over the 32 rows of this group
                    lo |= __shfl_xor(lo, off, 64);
                    hi |= __shfl_xor(hi, off, 64);
                }
                if ((row & 31) == 0) gm[(tb + u) * 4 + (row >> 5)] = ((uint64_t)hi << 32) | lo;
            }
        }
        __syncthreads();
    };
    auto tile_cols = [&](int t) -> uint64_t {
        uint64_t m = 0;
        for (int g = 0; g < NG; ++g) m |= gm[t * 4 + g];
        return m;
    };

    const bool one_segment = t1 - t0 <= kSeg;
    // Sweep 0: the entries that stay runs of 64 consecutive keys.  Sweep 1: the gathered ones, so
    // that the attention kernel meets a gathered entry (whose keys it must fetch before it can load
    // anything) only after it has other loads in flight.
    for (int sweep = 0; sweep < 2; ++sweep) {
        for (int seg = t0; seg < t1; seg += kSeg) {
            const int n = min(kSeg, t1 - seg);
            if (sweep == 0 || !one_segment) load_segment(seg, n);
            if (sweep == 0) {
                for (int t = 0; t < n; ++t) {
                    if (__popcll(tile_cols(t)) < min_cols) continue;   // also: nothing visible (min_cols >= 1)
                    const size_t e = (size_t)t0 + n_out;
                    if (row == 0) s.start[e] = k0s[t];
                    s.bitmaps[e * BM + row] = words[(size_t)t * BM + row];
                    ++n_out;
                }
                continue;
            }
            // classes (lo, hi): the groups that use a column span lo..hi
            for (int lo = 0; lo < NG; ++lo)
                for (int hi = lo; hi < NG; ++hi)
                    for (int t = 0; t < n; ++t) {
                        const uint64_t all = tile_cols(t);
                        if (all == 0 || __popcll(all) >= min_cols) continue;
                        uint64_t below = 0, above = 0;
                        for (int g = 0; g < lo; ++g) below |= gm[t * 4 + g];
                        for (int g = hi + 1; g < NG; ++g) above |= gm[t * 4 + g];
                        uint64_t colmask = (gm[t * 4 + lo] & ~below) & (gm[t * 4 + hi] & ~above);
                        if (colmask == 0) continue;
                        const uint64_t word = words[(size_t)t * BM + row];
                        const int k0 = k0s[t];
                        while (colmask) {                  // append this class's columns of the tile, ascending
                            const int bit = __ffsll((long long)colmask) - 1;
                            colmask &= colmask - 1;
                            if (fill == 0) {               // open a gathered entry: one per <= 64 columns,
                                tail_slot = (size_t)t0 + n_out;   // so never more entries than visible tiles
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
    const size_t lds = ((size_t)kSegWords + (size_t)kSegMax * 4) * sizeof(uint64_t);
    hipLaunchKernelGGL(build_schedule_kernel, dim3((unsigned)(H * nQB)), dim3(BM), lds, stream, row_ptr,
                       col_idx, bitmaps, nQB, Lq, Lk, BM, cap, causal, min_cols, s);
    return hipGetLastError();
}

}  // namespace ap
