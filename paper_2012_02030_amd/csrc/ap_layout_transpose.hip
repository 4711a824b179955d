// Transpose of a block-sparse layout: for every (head, block column) the stored tiles of that
// column in ascending block-row order.  The backward pass accumulates dK and dV per block
// column and walks this list.
//
// One thread per (head, block column): it looks its column up in every block row of the head
// (the columns of a block row ascend: binary search), first to count, then, after an exclusive
// scan of the counts, to fill.  The order is fixed by construction; no atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

namespace {

// position of column kb among col_idx[t0, t1), or -1
__device__ __forceinline__ int find_col(const int32_t* col_idx, int t0, int t1, int kb)
{
    int lo = t0, hi = t1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int c = col_idx[mid];
        if (c == kb) return mid;
        if (c < kb) lo = mid + 1;
        else hi = mid;
    }
    return -1;
}

template <bool FILL>
__global__ __launch_bounds__(256) void transpose_kernel(const int32_t* __restrict__ row_ptr,
                                                        const int32_t* __restrict__ col_idx, int H, int nQB,
                                                        int nKB, long long cap, int32_t* col_cnt_or_ptr,
                                                        int32_t* row_idx, int32_t* tile_idx)
{
    const int c = blockIdx.x * 256 + threadIdx.x;            // h * nKB + kb
    if (c >= H * nKB) return;
    const int h = c / nKB, kb = c - h * nKB;
    int n = 0;
    const int base = FILL ? col_cnt_or_ptr[c] : 0;
    for (int qb = 0; qb < nQB; ++qb) {
        const int r = h * nQB + qb;
        const int t0 = row_ptr[r];
        const int t1 = (int)min((long long)row_ptr[r + 1], cap);
        const int t = find_col(col_idx, t0, t1, kb);
        if (t >= 0) {
            if (FILL) {
                row_idx[base + n] = qb;
                tile_idx[base + n] = t;
            }
            ++n;
        }
    }
    if (!FILL) col_cnt_or_ptr[c + 1] = n;                    // shifted by one: the scan makes it a pointer
}

// In-place inclusive scan of ptr[1..n] (ptr[0] = 0) by one workgroup: counts -> pointers.
__global__ __launch_bounds__(1024) void scan_kernel(int32_t* ptr, int n)
{
    __shared__ int32_t part[1024];
    const int t = threadIdx.x;
    const int per = (n + 1023) / 1024;
    const int lo = 1 + t * per, hi = min(n + 1, lo + per);
    int32_t s = 0;
    for (int i = lo; i < hi; ++i) s += ptr[i];
    part[t] = s;
    __syncthreads();
    int32_t before = 0;
    for (int i = 0; i < t; ++i) before += part[i];
    if (t == 0) ptr[0] = 0;
    for (int i = lo; i < hi; ++i) {
        before += ptr[i];
        ptr[i] = before;
    }
}

}  // namespace

hipError_t launch_layout_transpose(const int32_t* row_ptr, const int32_t* col_idx, int H, int nQB,
                                   int nKB, long long cap, int32_t* col_ptr, int32_t* row_idx,
                                   int32_t* tile_idx, hipStream_t stream)
{
    const int ncol = H * nKB;
    const unsigned grid = (unsigned)((ncol + 255) / 256);
    hipLaunchKernelGGL(transpose_kernel<false>, dim3(grid), dim3(256), 0, stream, row_ptr, col_idx, H, nQB,
                       nKB, cap, col_ptr, row_idx, tile_idx);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, stream, col_ptr, ncol);
    hipLaunchKernelGGL(transpose_kernel<true>, dim3(grid), dim3(256), 0, stream, row_ptr, col_idx, H, nQB,
                       nKB, cap, col_ptr, row_idx, tile_idx);
    return hipGetLastError();
}

}  // namespace ap
