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
// last group; inside a class by tile, then ascending): an isolated connection is used by one
// query, so most gathered entries then concern one wavefront only and the other one skips them.
//
// One workgroup per block row, one thread per query row.  The bitmap words of a segment of tiles
// are brought into LDS with all loads in flight at once; the per-tile decisions are then taken with
// one lane per tile (column sets by OR over LDS, positions by prefix sums over the lanes), the
// gathered columns are listed in LDS in their final order, and only the assembly of each row's
// gathered words walks that list.  Every decision depends on OR-reductions of the row words only,
// so the emitted order is fixed: no atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

constexpr int kSegWords = 4096;                            // bitmap words of one segment (tiles x rows)
constexpr int kSegMax = 64;                                // at most this many tiles per segment (block_m = 64)

// inclusive prefix sum over the 64 lanes of a wavefront
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

// LDS (dynamic): words[t * (BM + 1) + row] (one word of padding per tile: a lane per tile then reads
// conflict-free), gm[t * 4 + g] = visible columns of 32-row group g of tile t, list[p] = tile << 6 | column
__global__ __launch_bounds__(128) void build_schedule_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const uint64_t* __restrict__ bitmaps, int nQB, int Lq, int Lk, int BM, long long cap,
    int causal, int min_cols, Schedule s)
{
    extern __shared__ uint64_t lds64[];
    const int kSeg = kSegWords / BM;                       // tiles per segment: 64 (block_m 64) or 32 (128)
    const int pitch = BM + 1;
    uint64_t* words = lds64;
    uint64_t* gm = lds64 + (size_t)kSegMax * 65;
    uint16_t* list = (uint16_t*)(gm + kSegMax * 4);
    __shared__ int32_t k0s[kSegMax];

    const int r = blockIdx.x;
    const int qb = r % nQB;
    const int row = threadIdx.x;                           // 0 .. BM-1
    const int lane = row & 63;
    const int NG = BM / 32;                                // 32-row groups (wavefronts of the attention kernel)
    const long long diag = (long long)qb * BM + row + ((long long)Lk - Lq);

    const int t0 = row_ptr[r];
    const int t1 = (int)min((long long)row_ptr[r + 1], cap);   // a truncated layout is never read past cap

    // Brings the (causally limited) words of tiles [seg, seg + n) into LDS and forms the visible
    // columns of every 32-row group of each.
    auto load_segment = [&](int seg, int n) {
        __syncthreads();                                   // previous use of the LDS arrays is over
        for (int t = row; t < n; t += BM) k0s[t] = col_idx[seg + t] * 64;
        __syncthreads();
        for (int tb = 0; tb < n; tb += 8) {
            uint64_t w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = tb + u < n ? bitmaps[(size_t)(seg + tb + u) * BM + row] : 0ull;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (tb + u >= n) break;
                uint64_t word = w[u];
                if (causal) {
                    const long long lim = diag - (long long)k0s[tb + u];
                    if (lim < 0) word = 0;
                    else if (lim < 63) word &= (2ull << lim) - 1ull;
                }
                words[(size_t)(tb + u) * pitch + row] = word;
            }
        }
        __syncthreads();
        for (int pair = row; pair < n * NG; pair += BM) {  // (tile, group): OR of its 32 row words
            const int t = pair / NG, g = pair % NG;
            uint64_t m = 0;
#pragma unroll 8
            for (int rr = 0; rr < 32; ++rr) m |= words[(size_t)t * pitch + 32 * g + rr];
            gm[t * 4 + g] = m;
        }
        __syncthreads();
    };
    // what lane l (< n) of every wavefront knows about tile l of the segment
    struct Tile {
        uint64_t g[4];
        bool cons, gath;
    };
    auto tile_info = [&](int n) -> Tile {
        Tile ti;
        uint64_t all = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            ti.g[g] = (lane < n && g < NG) ? gm[lane * 4 + g] : 0ull;
            all |= ti.g[g];
        }
        const int nc = __popcll(all);
        ti.cons = nc > 0 && nc >= min_cols;
        ti.gath = nc > 0 && nc < min_cols;
        return ti;
    };

    const bool one_segment = t1 - t0 <= kSeg;
    int n_cons = 0;                                        // consecutive entries emitted so far
    // Sweep 0: the entries that stay runs of 64 consecutive keys, in tile order.
    for (int seg = t0; seg < t1; seg += kSeg) {
        const int n = min(kSeg, t1 - seg);
        load_segment(seg, n);
        const Tile ti = tile_info(n);
        unsigned long long cm = __ballot(ti.cons);         // the same in every wavefront
        while (cm) {
            const int t = __ffsll((long long)cm) - 1;
            cm &= cm - 1;
            const size_t e = (size_t)t0 + n_cons;
            if (row == 0) s.start[e] = k0s[t];
            s.bitmaps[e * BM + row] = words[(size_t)t * pitch + row];
            ++n_cons;
        }
    }
    // Sweep 1: the gathered entries, so that the attention kernel meets a gathered entry (whose keys
    // it must fetch before it can load anything) only after it has other loads in flight.  Their
    // slots follow the consecutive ones: column number p of the block row's gathered stream sits
    // in slot p % 64 of entry t0 + n_cons + p / 64.
    const size_t first = (size_t)t0 + n_cons;
    long long stream = 0;                                  // gathered columns emitted so far
    uint64_t tail_word = 0;                                // this row's bits of the open gathered entry
    for (int seg = t0; seg < t1; seg += kSeg) {
        const int n = min(kSeg, t1 - seg);
        if (!one_segment) load_segment(seg, n);
        const Tile ti = tile_info(n);
        // classes (lo, hi): the groups that use a column span lo..hi; the columns are listed class
        // by class, tile by tile, ascending
        int total = 0;
        for (int lo = 0; lo < NG; ++lo)
            for (int hi = lo; hi < NG; ++hi) {
                uint64_t below = 0, above = 0, glo = 0, ghi = 0;
#pragma unroll
                for (int g = 0; g < 4; ++g) {              // compile-time register indices
                    if (g < lo) below |= ti.g[g];
                    if (g > hi) above |= ti.g[g];
                    if (g == lo) glo = ti.g[g];
                    if (g == hi) ghi = ti.g[g];
                }
                uint64_t cmask = ti.gath ? ((glo & ~below) & (ghi & ~above)) : 0ull;
                const int cnt = __popcll(cmask);
                const int incl = wave_inclusive_scan(cnt, lane);
                int pos = total + incl - cnt;
                if (row < 64) {                            // the first wavefront writes the list
                    while (cmask) {
                        const int bit = __ffsll((long long)cmask) - 1;
                        cmask &= cmask - 1;
                        list[pos++] = (uint16_t)((lane << 6) | bit);
                    }
                }
                total += __shfl(incl, 63, 64);
            }
        __syncthreads();
        // keys and kinds of the gathered slots of this segment, in parallel
        for (int p = row; p < total; p += BM) {
            const int it = list[p];
            const long long gp = stream + p;
            s.cols[(first + (size_t)(gp >> 6)) * 64 + (gp & 63)] = k0s[it >> 6] + (it & 63);
            if ((gp & 63) == 0) s.start[first + (size_t)(gp >> 6)] = -1;
        }
        // every row assembles its words by walking the list
        int fill = (int)(stream & 63);
        for (int p = 0; p < total; ++p) {
            const int it = list[p];
            const uint64_t word = words[(size_t)(it >> 6) * pitch + row];
            tail_word |= ((word >> (it & 63)) & 1ull) << fill;
            if (++fill == 64) {
                s.bitmaps[(first + (size_t)((stream + p) >> 6)) * BM + row] = tail_word;
                tail_word = 0;
                fill = 0;
            }
        }
        stream += total;
    }
    const int fill = (int)(stream & 63);
    if (fill > 0) {                                        // last, partly filled gathered entry
        const size_t e = first + (size_t)(stream >> 6);
        for (int c = fill + row; c < 64; c += BM) s.cols[e * 64 + c] = Lk;   // empty slot: reads as zeros
        s.bitmaps[e * BM + row] = tail_word;
    }
    if (row == 0) s.cnt[r] = n_cons + (int)((stream + 63) >> 6);
}

}  // namespace

hipError_t launch_build_schedule(const int32_t* row_ptr, const int32_t* col_idx,
                                 const uint64_t* bitmaps, int H, int Lq, int Lk, int BM,
                                 long long cap, int causal, int min_cols, const Schedule& s,
                                 hipStream_t stream)
{
    const int nQB = (Lq + BM - 1) / BM;
    // words (padded), group column sets, column list
    const size_t lds = ((size_t)kSegMax * 65 + (size_t)kSegMax * 4) * sizeof(uint64_t) +
                       (size_t)kSegMax * 64 * sizeof(uint16_t);
    hipLaunchKernelGGL(build_schedule_kernel, dim3((unsigned)(H * nQB)), dim3(BM), lds, stream, row_ptr,
                       col_idx, bitmaps, nQB, Lq, Lk, BM, cap, causal, min_cols, s);
    return hipGetLastError();
}

}  // namespace ap
