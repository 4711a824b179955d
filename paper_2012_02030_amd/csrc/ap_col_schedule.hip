// Column schedule: the visit schedule of the backward pass's dK/dV kernel, a re-packing of the
// transposed layout.  For every (head, block column) the stored tiles are walked in ascending
// block-row order; a tile in which at least `min_rows` query rows hold a visible kept entry stays
// a run of 64 consecutive queries, the rows of all other tiles that hold one are packed, in
// ascending order, into gathered entries of 64 arbitrary queries.  Every entry carries, per
// query slot, the 64-bit word of kept keys inside this block column with the causal limit
// folded in.  Same structure as the row schedule with the roles of rows and columns swapped.
//
// One wavefront per block column, one lane per tile row; all control flow depends on ballots
// only, so the emitted order is fixed: no atomics.  A second kernel appends, behind the entry
// counts, the order in which the dK/dV kernel should visit the block columns of each head.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

__global__ __launch_bounds__(64) void build_col_schedule_kernel(
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ row_idx,
    const int32_t* __restrict__ tile_idx, const uint64_t* __restrict__ bitmaps, int nKB, int Lq, int Lk,
    int causal, int min_rows, Schedule s)
{
    const int c = blockIdx.x;
    const int kb = c % nKB;
    const int lane = threadIdx.x;
    const long long off = (long long)Lk - Lq;
    const int c0 = col_ptr[c], c1 = col_ptr[c + 1];
    int n_out = 0;                                           // entry slots handed out so far
    int fill = 0;                                            // query slots used in the open gathered entry
    size_t open = 0;                                         // its position
    for (int pass = 0; pass < 2; ++pass) {
        for (int ci = c0; ci < c1; ++ci) {
            const int q0 = row_idx[ci] * 64;
            uint64_t word = bitmaps[(size_t)tile_idx[ci] * 64 + lane];
            if (causal) {
                const long long lim = (long long)q0 + lane + off - (long long)kb * 64;
                if (lim < 0) word = 0;
                else if (lim < 63) word &= (2ull << lim) - 1ull;
            }
            const unsigned long long rows = __ballot(word != 0);
            const int nrows = __popcll(rows);
            if (nrows == 0) continue;                        // nothing visible
            const bool consecutive = nrows >= min_rows;
            if (consecutive != (pass == 0)) continue;
            if (consecutive) {
                const size_t e = (size_t)c0 + n_out++;
                if (lane == 0) s.start[e] = q0;
                s.bitmaps[e * 64 + lane] = word;
                continue;
            }
            if (fill == 0) open = (size_t)c0 + n_out++;      // open a gathered entry
            const bool spill = fill + nrows > 64;            // the rows do not all fit into it
            const size_t next = spill ? (size_t)c0 + n_out++ : 0;
            if (word != 0) {
                const int slot = fill + __popcll(rows & ((1ull << lane) - 1ull));
                const size_t e = slot < 64 ? open : next;
                s.cols[e * 64 + (slot & 63)] = q0 + lane;
                s.bitmaps[e * 64 + (slot & 63)] = word;
            }
            if (lane == 0) {
                s.start[open] = -1;
                if (spill) s.start[next] = -1;
            }
            fill += nrows;
            if (fill >= 64) {                                // the open entry is complete
                fill -= 64;
                open = next;
            }
        }
    }
    if (fill > 0 && lane >= fill) {                          // empty slots of the last gathered entry
        s.cols[open * 64 + lane] = Lq;                       // beyond the last query: reads as zeros
        s.bitmaps[open * 64 + lane] = 0;
    }
    if (lane == 0) s.cnt[c] = n_out;
}

// Visiting order of the block columns of one head: columns with at least twice the head's mean
// number of entries ("heavy": their workgroups run longest and should start first) in ascending
// order, then the others in ascending order.  One wavefront per head.
//   order  [H*nKB]  block column at each position      n_heavy [H]  number of heavy columns
__global__ __launch_bounds__(64) void col_order_kernel(const int32_t* __restrict__ cnt, int nKB,
                                                       int32_t* __restrict__ order, int32_t* __restrict__ n_heavy)
{
    const int h = blockIdx.x;
    const int lane = threadIdx.x;
    const int32_t* c = cnt + (size_t)h * nKB;
    long long sum = 0;
    for (int k = lane; k < nKB; k += 64) sum += c[k];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const long long limit = (2 * sum + nKB - 1) / nKB;       // ceil(2 * mean)
    int pos = 0;
    for (int pass = 0; pass < 2; ++pass) {
        for (int k0 = 0; k0 < nKB; k0 += 64) {
            const int k = k0 + lane;
            const bool heavy = k < nKB && c[k] >= limit && c[k] > 1;
            const bool take = k < nKB && heavy == (pass == 0);
            const unsigned long long m = __ballot(take);
            if (take) order[(size_t)h * nKB + pos + __popcll(m & ((1ull << lane) - 1ull))] = k;
            pos += __popcll(m);
        }
        if (pass == 0 && lane == 0) n_heavy[h] = pos;
    }
}

}  // namespace

hipError_t launch_build_col_schedule(const int32_t* col_ptr, const int32_t* row_idx, const int32_t* tile_idx,
                                     const uint64_t* bitmaps, int H, int Lq, int Lk, int causal,
                                     int min_rows, const Schedule& s, hipStream_t stream)
{
    const int nKB = (Lk + 63) / 64;
    hipLaunchKernelGGL(build_col_schedule_kernel, dim3((unsigned)(H * nKB)), dim3(64), 0, stream, col_ptr,
                       row_idx, tile_idx, bitmaps, nKB, Lq, Lk, causal, min_rows, s);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int32_t* order = s.cnt + (size_t)H * nKB;                // the count array carries the visiting order
    hipLaunchKernelGGL(col_order_kernel, dim3((unsigned)H), dim3(64), 0, stream, s.cnt, nKB, order,
                       order + (size_t)H * nKB);
    return hipGetLastError();
}

}  // namespace ap
