// Layout pass: element mask -> block rows / block columns / per-tile element bitmaps.
//
// The paper's hardware section (Section 9.2) runs Attention Pruning on block-sparse kernels;
// the mask itself is the element-wise threshold of Eq. (2).  This pass keeps both: a tile is
// stored iff its window holds a kept entry, and every stored tile carries its element bitmap.
//
// Kernels, all bound by the single read of the mask from HBM:
//   strip_scan 64-key windows (the attention kernels' shape): one wavefront per strip of 16
//              windows of a block row; every mask row of the strip is one contiguous read of
//              1024 entries (16 per lane), packed to bits in registers, assembled into row words,
//              staged in LDS and written to a dense scratch array as whole windows, one non-empty
//              flag per window.  The source is the byte mask, or (Eq. (2) evaluated on the fly)
//              the fp32 mean map with the layer's threshold: kept iff not (value < tau), and
//              visible if the attention is causal
//   tile_scan  any other window shape: one wavefront per window
//   row_count  one wavefront per block row: ballot + popcount over the flags
//   row_scan   exclusive prefix sum of the per-row counts (one workgroup) -> row_ptr, nnz
//   compact    one workgroup per block row: ballot rank gives every kept window its position
//              (ascending block column, no atomics), then its wavefronts copy the bitmaps
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ap_internal.h"

namespace ap {

// 4 mask bytes -> 4 bits (bit k = byte k nonzero)
__device__ __forceinline__ uint32_t nonzero_bytes_to_bits(uint32_t x)
{
    // high bit of every nonzero byte
    uint32_t y = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;
    // gather bits 7,15,23,31 into the top nibble
    return ((y >> 7) * 0x10204080u) >> 28;
}

// One wavefront per window.  lanes_per_row = BN/16 lanes cover one mask row of the window with
// one 16-byte load each; 64/lanes_per_row rows are covered per pass.
__global__ __launch_bounds__(256) void tile_scan_kernel(
    const uint8_t* __restrict__ mask, long long stride_h, long long stride_row, int H, int Lq, int Lk,
    int BM, int BN, int nQB, int nKB, int vec_ok, uint8_t* __restrict__ flags,
    uint64_t* __restrict__ dense /* may be null */)
{
    const int lane = threadIdx.x & 63;
    const long long tile = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long long n_tiles = (long long)H * nQB * nKB;
    if (tile >= n_tiles) return;                       // whole wavefront leaves together
    const int kb = (int)(tile % nKB);
    const int qb = (int)((tile / nKB) % nQB);
    const int h = (int)(tile / ((long long)nKB * nQB));

    const int W = (BN + 63) >> 6;
    const int lpr = BN >> 4;                           // lanes per row: 1, 2, 4 or 8
    const int rpp = 64 / lpr;                          // rows per pass
    const int seg = lane % lpr;
    const int rsub = lane / lpr;
    const int j0 = kb * BN + seg * 16;                 // first column this lane covers

    bool any = false;
    for (int r0 = 0; r0 < BM; r0 += rpp) {
        const int rr = r0 + rsub;
        const int i = qb * BM + rr;
        uint32_t bits = 0;
        if (rr < BM && i < Lq && j0 < Lk) {
            const uint8_t* p = mask + (size_t)h * stride_h + (size_t)i * stride_row + j0;
            if (vec_ok) {                              // Lk and the row pitch % 16 == 0: the 16 bytes are in range and aligned
                const uint4 v = *reinterpret_cast<const uint4*>(p);
                bits = nonzero_bytes_to_bits(v.x) | (nonzero_bytes_to_bits(v.y) << 4) |
                       (nonzero_bytes_to_bits(v.z) << 8) | (nonzero_bytes_to_bits(v.w) << 12);
            } else {
                for (int c = 0; c < 16; ++c)
                    if (j0 + c < Lk && p[c] != 0) bits |= 1u << c;
            }
        }
        // assemble the 64-bit word from the (up to) 4 lanes that share it
        uint64_t word = (uint64_t)bits << (16 * (seg & 3));
        if (lpr >= 2) word |= __shfl_xor(word, 1, 64);
        if (lpr >= 4) word |= __shfl_xor(word, 2, 64);
        any |= (__ballot(word != 0) != 0);
        if (dense && rr < BM && (seg & 3) == 0)
            dense[((size_t)tile * BM + rr) * W + (seg >> 2)] = word;
    }
    if (lane == 0) flags[tile] = any ? 1 : 0;
}

// 16 entries of one mask row -> 16 bits.  Byte mask: nonzero = kept.
__device__ __forceinline__ uint32_t keep_bits16(const uint8_t* p, int n_valid, bool vec)
{
    if (vec && n_valid >= 16) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        return nonzero_bytes_to_bits(v.x) | (nonzero_bytes_to_bits(v.y) << 4) |
               (nonzero_bytes_to_bits(v.z) << 8) | (nonzero_bytes_to_bits(v.w) << 12);
    }
    uint32_t bits = 0;
    for (int c = 0; c < 16; ++c)
        if (c < n_valid && p[c] != 0) bits |= 1u << c;
    return bits;
}
// Mean map with threshold (Eq. (2)): pruned iff value < tau, so kept iff not (value < tau).
__device__ __forceinline__ uint32_t keep_bits16(const float* p, int n_valid, bool vec, float tau)
{
    uint32_t bits = 0;
    if (vec && n_valid >= 16) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = *reinterpret_cast<const float4*>(p + 4 * q);
            bits |= (uint32_t)(!(v.x < tau)) << (4 * q) | (uint32_t)(!(v.y < tau)) << (4 * q + 1) |
                    (uint32_t)(!(v.z < tau)) << (4 * q + 2) | (uint32_t)(!(v.w < tau)) << (4 * q + 3);
        }
        return bits;
    }
    for (int c = 0; c < 16; ++c)
        if (c < n_valid && !(p[c] < tau)) bits |= 1u << c;
    return bits;
}

// One wavefront per (head, block row, strip of 16 windows of 64 keys).  Lane l covers columns
// 1024 * strip + 16 * l .. + 15 of every row of the block row: a wavefront reads 1024 consecutive
// entries of one mask row at a time.  Four lanes share a 64-bit row word.  The words of the
// strip are staged in LDS as [window][row] and written out window by window (contiguous).
// causal_off = Lk - Lq if entries j > i + (Lk - Lq) are never kept (map source only), else a
// value no column reaches.
template <typename SRC>
__global__ __launch_bounds__(256) void strip_scan_kernel(
    const SRC* __restrict__ src, const float* __restrict__ tau_ptr, long long stride_h, long long stride_row,
    int H, int Lq, int Lk, int BM, int nQB, int nKB, long long causal_off, int vec_ok,
    uint8_t* __restrict__ flags, uint64_t* __restrict__ dense /* may be null */)
{
    extern __shared__ uint64_t stage_all[];                  // [4 wavefronts][16 windows][BM rows]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int strips = (nKB + 15) >> 4;
    const long long unit = (long long)blockIdx.x * 4 + wave;
    const long long n_units = (long long)H * nQB * strips;
    if (unit >= n_units) return;                             // whole wavefront leaves together; no barrier below
    const int strip = (int)(unit % strips);
    const int qb = (int)((unit / strips) % nQB);
    const int h = (int)(unit / ((long long)strips * nQB));
    uint64_t* stage = stage_all + (size_t)wave * 16 * BM;

    const int col0 = strip * 1024 + lane * 16;               // first column this lane covers
    const int win = lane >> 2, quarter = lane & 3;           // window inside the strip, 16-column piece inside its words
    const int kb = strip * 16 + win;
    float tau = 0.f;
    if constexpr (sizeof(SRC) == 4) tau = *tau_ptr;
    const SRC* base = src + (size_t)h * stride_h + col0;

    // rows in flight per lane: the whole kernel is one round of wavefronts, so its duration is the
    // number of dependent memory round trips of one wavefront (16 KB in flight per wavefront)
    constexpr int RB = sizeof(SRC) == 1 ? 16 : 4;
    uint64_t any = 0;
    for (int r0 = 0; r0 < BM; r0 += RB) {
        uint32_t bits[RB];
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int rr = r0 + u;
            const long long i = (long long)qb * BM + rr;
            // columns this lane may keep in row i: inside the mask, and visible if causal
            long long lim = (long long)Lk - col0;
            if (causal_off + i + 1 - col0 < lim) lim = causal_off + i + 1 - col0;
            const int n_valid = (i < Lq && lim > 0) ? (int)(lim < 16 ? lim : 16) : 0;
            // the vector path reads all 16 entries: they must lie inside the row
            const bool vec = vec_ok && col0 + 16 <= Lk;
            uint32_t b = 0;
            if (n_valid > 0) {
                const SRC* p = base + (size_t)i * stride_row;
                if constexpr (sizeof(SRC) == 4) b = keep_bits16(p, vec ? 16 : n_valid, vec, tau);
                else b = keep_bits16(p, vec ? 16 : n_valid, vec);
                if (n_valid < 16) b &= (1u << n_valid) - 1u;
            }
            bits[u] = b;
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            uint64_t word = (uint64_t)bits[u] << (16 * quarter);
            word |= __shfl_xor(word, 1, 64);
            word |= __shfl_xor(word, 2, 64);
            any |= word;
            if (dense && quarter == 0) stage[win * BM + r0 + u] = word;
        }
    }
    if (quarter == 0 && kb < nKB) flags[((size_t)h * nQB + qb) * nKB + kb] = any != 0 ? 1 : 0;
    if (dense) {
        // same wavefront reads back what it wrote: LDS ordering only
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const int n_win = min(16, nKB - strip * 16);
        uint64_t* dst = dense + (((size_t)h * nQB + qb) * nKB + (size_t)strip * 16) * BM;
        for (int idx = lane; idx < n_win * BM; idx += 64) dst[idx] = stage[idx];
    }
}

__global__ __launch_bounds__(256) void row_count_kernel(
    const uint8_t* __restrict__ flags, int n_rows, int nKB, int32_t* __restrict__ counts)
{
    const int lane = threadIdx.x & 63;
    const long long r = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    int cnt = 0;
    for (int k0 = 0; k0 < nKB; k0 += 64) {
        const int kb = k0 + lane;
        const bool f = kb < nKB && flags[(size_t)r * nKB + kb] != 0;
        cnt += __popcll(__ballot(f));
    }
    if (lane == 0) counts[r] = cnt;
}

// Exclusive prefix sum over counts[0..n) by one workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void row_scan_kernel(
    const int32_t* __restrict__ counts, int n_rows, int32_t* __restrict__ row_ptr,
    int64_t* __restrict__ nnz_out)
{
    __shared__ long long part[1024];
    const int t = threadIdx.x;
    const int per = (n_rows + 1023) / 1024;
    const int lo = t * per;
    const int hi = min(lo + per, n_rows);
    long long s = 0;
    for (int i = lo; i < hi; ++i) s += counts[i];
    part[t] = s;
    __syncthreads();
    // Hillis-Steele inclusive scan of the 1024 partial sums
    for (int off = 1; off < 1024; off <<= 1) {
        long long v = (t >= off) ? part[t - off] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    long long run = part[t] - s;                       // exclusive prefix of this thread's chunk
    for (int i = lo; i < hi; ++i) {
        row_ptr[i] = (int32_t)run;
        run += counts[i];
    }
    if (t == 1023) {
        row_ptr[n_rows] = (int32_t)part[1023];
        if (nnz_out) *nnz_out = part[1023];
    }
}

__global__ __launch_bounds__(256) void compact_kernel(
    const uint8_t* __restrict__ flags, const uint64_t* __restrict__ dense,
    const int32_t* __restrict__ row_ptr, int n_rows, int nKB, int words_per_tile,
    int32_t* __restrict__ col_idx, uint64_t* __restrict__ bitmaps, long long cap)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;                       // the four wavefronts take the kept windows in turn
    const long long r = blockIdx.x;
    long long base = row_ptr[r];
    for (int k0 = 0; k0 < nKB; k0 += 64) {
        const int kb = k0 + lane;
        const bool f = kb < nKB && flags[(size_t)r * nKB + kb] != 0;
        const unsigned long long bal = __ballot(f);
        const int rank = __popcll(bal & ((1ull << lane) - 1ull));
        if (wave == 0 && f && base + rank < cap) col_idx[base + rank] = kb;
        unsigned long long rest = bal;
        long long pos = base;
        while (rest) {
            const int src_lane = __ffsll((long long)rest) - 1;
            rest &= rest - 1;
            if (pos < cap && ((pos - base) & 3) == wave) {
                const uint64_t* src = dense + ((size_t)r * nKB + (k0 + src_lane)) * words_per_tile;
                uint64_t* dst = bitmaps + (size_t)pos * words_per_tile;
                for (int w = lane; w < words_per_tile; w += 64) dst[w] = src[w];
            }
            ++pos;
        }
        base += __popcll(bal);
    }
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool layout_shape_ok(int H, int Lq, int Lk, int BM, int BN)
{
    if (H <= 0 || Lq <= 0 || Lk <= 0) return false;
    if (!(BM == 16 || BM == 32 || BM == 64 || BM == 128)) return false;
    if (!(BN == 16 || BN == 32 || BN == 64 || BN == 128)) return false;
    const long long nQB = (Lq + BM - 1) / BM, nKB = (Lk + BN - 1) / BN;
    return (long long)H * nQB * nKB < 2147483647LL;
}

void layout_workspace_plan(int H, int Lq, int Lk, int BM, int BN, size_t* flags_off,
                           size_t* counts_off, size_t* dense_off, size_t* total)
{
    const size_t nQB = (Lq + BM - 1) / BM, nKB = (Lk + BN - 1) / BN, W = (BN + 63) / 64;
    const size_t n_rows = (size_t)H * nQB, n_tiles = n_rows * nKB;
    size_t off = 0;
    *flags_off = off;  off = align_up(off + n_tiles, 16);
    *counts_off = off; off = align_up(off + n_rows * sizeof(int32_t), 16);
    *dense_off = off;  off = align_up(off + n_tiles * BM * W * sizeof(uint64_t), 16);
    *total = off;
}

template <typename SRC>
static hipError_t launch_build_layout_any(const SRC* src, const float* tau, long long causal_off, long long stride_h,
                                          long long stride_row, int H, int Lq, int Lk, int BM, int BN,
                                          int32_t* row_ptr, int32_t* col_idx, uint64_t* bitmaps, long long cap,
                                          int64_t* nnz_out, void* workspace, hipStream_t stream)
{
    const int nQB = (Lq + BM - 1) / BM, nKB = (Lk + BN - 1) / BN, W = (BN + 63) / 64;
    const int n_rows = H * nQB;
    const long long n_tiles = (long long)n_rows * nKB;
    size_t flags_off, counts_off, dense_off, total;
    layout_workspace_plan(H, Lq, Lk, BM, BN, &flags_off, &counts_off, &dense_off, &total);
    uint8_t* flags = (uint8_t*)workspace + flags_off;
    int32_t* counts = (int32_t*)((uint8_t*)workspace + counts_off);
    uint64_t* dense = col_idx ? (uint64_t*)((uint8_t*)workspace + dense_off) : nullptr;
    // 16 entries per load
    const int vec_ok = ((Lk * sizeof(SRC)) % 16 == 0) && ((stride_row * sizeof(SRC)) % 16 == 0) &&
                       ((stride_h * sizeof(SRC)) % 16 == 0) && (((uintptr_t)src & 15) == 0);

    const int waves_per_block = 4;
    const unsigned row_blocks = (unsigned)((n_rows + waves_per_block - 1) / waves_per_block);

    if (BN == 64) {                                          // block_m is a multiple of 16
        const long long units = (long long)n_rows * ((nKB + 15) / 16);
        const size_t lds = (size_t)4 * 16 * BM * sizeof(uint64_t);
        hipLaunchKernelGGL(strip_scan_kernel<SRC>, dim3((unsigned)((units + 3) / 4)), dim3(256), lds, stream, src, tau,
                           stride_h, stride_row, H, Lq, Lk, BM, nQB, nKB, causal_off, vec_ok, flags, dense);
    } else if constexpr (sizeof(SRC) == 1) {
        const unsigned tile_blocks = (unsigned)((n_tiles + waves_per_block - 1) / waves_per_block);
        hipLaunchKernelGGL(tile_scan_kernel, dim3(tile_blocks), dim3(64 * waves_per_block), 0, stream,
                           src, stride_h, stride_row, H, Lq, Lk, BM, BN, nQB, nKB, vec_ok, flags, dense);
    } else {
        return hipErrorInvalidValue;                         // the map source is scanned in 64-key windows only
    }
    hipLaunchKernelGGL(row_count_kernel, dim3(row_blocks), dim3(64 * waves_per_block), 0, stream,
                       flags, n_rows, nKB, counts);
    hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(1024), 0, stream, counts, n_rows, row_ptr,
                       nnz_out);
    if (col_idx)
        hipLaunchKernelGGL(compact_kernel, dim3((unsigned)n_rows), dim3(256), 0, stream,
                           flags, dense, row_ptr, n_rows, nKB, BM * W, col_idx, bitmaps, cap);
    return hipGetLastError();
}

hipError_t launch_build_layout(const uint8_t* mask, long long stride_h, long long stride_row, int H,
                               int Lq, int Lk, int BM, int BN, int32_t* row_ptr, int32_t* col_idx, uint64_t* bitmaps,
                               long long cap, int64_t* nnz_out, void* workspace,
                               hipStream_t stream)
{
    // no column reaches the limit: every entry of the byte mask counts
    return launch_build_layout_any<uint8_t>(mask, nullptr, (long long)1 << 40, stride_h, stride_row, H, Lq, Lk, BM,
                                            BN, row_ptr, col_idx, bitmaps, cap, nnz_out, workspace, stream);
}

hipError_t launch_build_layout_from_map(const float* abar, const float* tau, int causal, int H, int Lq, int Lk,
                                        int BM, int BN, int32_t* row_ptr, int32_t* col_idx, uint64_t* bitmaps,
                                        long long cap, int64_t* nnz_out, void* workspace, hipStream_t stream)
{
    const long long causal_off = causal ? (long long)Lk - Lq : (long long)1 << 40;
    return launch_build_layout_any<float>(abar, tau, causal_off, (long long)Lq * Lk, Lk, H, Lq, Lk, BM, BN, row_ptr,
                                          col_idx, bitmaps, cap, nnz_out, workspace, stream);
}

}  // namespace ap
