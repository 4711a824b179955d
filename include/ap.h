/*
 * ap.h -- C ABI of the MI355X (gfx950) masked-attention library for Attention Pruning (AP).
 *
 * AP fixes one global sparseness mask per (layer, head): entries of the attention matrix
 * whose dataset-averaged weight falls below a percentile threshold are pruned (paper,
 * Section 3.2, Eq. (1) and Eq. (2)), and attention is then computed as
 *
 *     A~ = softmax( (Q K^T + M_p) / sqrt(d_k) ) V              (Section 3.2, masked equation)
 *
 * with M_p = 0 on kept entries and -infinity on pruned ones.  The mask has no batch index.
 * This library evaluates that expression only where the mask is set.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer.  The library allocates and frees nothing and keeps no
 *     state between calls.
 *   - Every call enqueues work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and returns without synchronising.
 *   - Errors are return codes; nothing throws or aborts.  Arguments are validated on the
 *     host before anything is launched, so a call that returns AP_ERR_INVALID_ARG or
 *     AP_ERR_UNSUPPORTED has touched no device memory.
 *   - Results are deterministic: the layout is bit-identical from run to run, and O is
 *     bitwise reproducible for fixed inputs (fixed tile order, no atomics).
 */
#ifndef AP_H
#define AP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ap_status {
    AP_OK = 0,
    AP_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, misaligned pointer or stride, ...  */
    AP_ERR_UNSUPPORTED = -2, /* valid request outside what the kernels implement (D, tile shape)   */
    AP_ERR_CAPACITY = -3,    /* a caller-provided buffer is smaller than the stated requirement     */
    AP_ERR_HIP = -4          /* the HIP runtime refused a launch or no GPU is present               */
} ap_status;

typedef enum ap_dtype {
    AP_F32 = 0, /* IEEE binary32 in and out, fp32 arithmetic                                        */
    AP_BF16 = 1 /* bfloat16 in and out, bf16 matrix-core products with fp32 accumulation            */
} ap_dtype;

/* Human-readable name of a status code (host pointer to a static string). */
const char *ap_status_string(ap_status s);

/* ---------------------------------------------------------------------------------------------
 * Layout: element mask -> block-sparse layout.
 *
 * The paper's hardware section (Section 9.2) runs AP on block-sparse kernels, i.e. the mask of
 * Eq. (2) is organised in blocks.  Here a block ("tile") is block_m query rows by block_n key
 * columns, and each stored tile carries the element bitmap of its window, so the element
 * mask of Eq. (2) is represented exactly rather than rounded to blocks.
 *
 *   nQB = ceil(Lq / block_m), nKB = ceil(Lk / block_n), W = ceil(block_n / 64).
 *   A tile (h, qb, kb) is stored iff any mask byte inside its window (clipped to Lq x Lk) is
 *   nonzero.  Block rows are numbered r = h * nQB + qb.
 *
 *   row_ptr [H*nQB + 1]  int32   exclusive prefix sum of stored tiles per block row; row_ptr[0] = 0
 *   col_idx [nnz]        int32   kb of each stored tile, ascending inside a block row
 *   bitmaps [nnz*block_m*W] uint64  word (t, rr, w): bit c%64 of word w = c/64 is
 *                                mask[h, qb*block_m + rr, kb*block_n + c] != 0; bits whose
 *                                row or column lies outside the mask are 0
 *
 * Supported: block_m in {16, 32, 64, 128}, block_n in {16, 32, 64, 128}; H*nQB*nKB < 2^31.
 * ------------------------------------------------------------------------------------------- */

/* Upper bound H*nQB*nKB on the number of stored tiles (so buffers can be sized without a
 * device round trip).  Returns -1 for invalid arguments. */
int64_t ap_layout_max_tiles(int H, int Lq, int Lk, int block_m, int block_n);

/* Bytes of device scratch that ap_build_layout needs for these sizes (0 for invalid arguments). */
size_t ap_layout_workspace_bytes(int H, int Lq, int Lk, int block_m, int block_n);

/*
 * Build the layout of `mask` (uint8 [H, Lq, Lk], row-major, any nonzero byte = kept).
 *
 *   row_ptr      out, int32 [H*nQB + 1]
 *   col_idx      out, int32 [cap]; may be NULL together with bitmaps to obtain only row_ptr
 *                and nnz_out (count-only use: read nnz_out, allocate exactly, call again)
 *   bitmaps      out, uint64 [cap * block_m * W], 8-byte aligned
 *   cap          number of tiles col_idx/bitmaps have room for.  Tiles whose position is
 *                >= cap are counted but not written: the call stays asynchronous, so the
 *                caller compares *nnz_out with cap after synchronising.  Passing
 *                cap >= ap_layout_max_tiles(...) can never truncate.
 *   nnz_out      out, device int64: total number of stored tiles (= row_ptr[H*nQB]); may be NULL
 *   workspace    device scratch of at least ap_layout_workspace_bytes(...) bytes, 8-byte aligned;
 *                contents are undefined afterwards
 *
 * Returns AP_ERR_CAPACITY if workspace_bytes is too small, AP_ERR_INVALID_ARG / AP_ERR_UNSUPPORTED
 * for bad sizes or pointers, AP_ERR_HIP if a launch fails.
 */
ap_status ap_build_layout(const uint8_t *mask, int H, int Lq, int Lk, int block_m, int block_n,
                          int32_t *row_ptr, int32_t *col_idx, uint64_t *bitmaps, int64_t cap,
                          int64_t *nnz_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same for the top-left Lq x Lk corner of a stored mask [H, Lq_stored, Lk_stored] (Section 6:
 * sequence lengths vary across a data set while the mask of a layer and head is fixed, so a
 * shorter sequence uses the corner of the mask that covers it).  The result is the layout that
 * ap_build_layout would produce for a contiguous copy of that corner; nothing is copied.
 * Lq <= Lq_stored, Lk <= Lk_stored; workspace as for (H, Lq, Lk).
 */
ap_status ap_build_layout_cropped(const uint8_t *mask, int H, int Lq_stored, int Lk_stored, int Lq,
                                  int Lk, int block_m, int block_n, int32_t *row_ptr, int32_t *col_idx,
                                  uint64_t *bitmaps, int64_t cap, int64_t *nnz_out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * The layout straight from the mean attention map (Section 3.2, Eq. (2)): the strict comparison
 * with the layer's threshold is evaluated inside the scan, so the byte mask is never written or
 * read.  The result is bit for bit the layout that ap_build_layout produces for the mask that
 * ap_prune_mask writes for the same map and threshold:
 *
 *     kept(h,i,j)  <=>  not (abar[h,i,j] < tau)  and  (not causal or j <= i + (Lk - Lq))
 *
 *   abar          float [H, Lq, Lk] contiguous (as for ap_prune_mask; entries that causality hides
 *                 may hold anything, they are never kept)
 *   tau           device pointer to the threshold, e.g. ap_prune_mask's tau_out (that call
 *                 accepts mask = NULL to compute the threshold only); +infinity keeps nothing
 *   everything else as in ap_build_layout, workspace included; block_n must be 64
 */
ap_status ap_build_layout_from_map(const float *abar, const float *tau, int H, int Lq, int Lk, int causal,
                                   int block_m, int block_n, int32_t *row_ptr, int32_t *col_idx,
                                   uint64_t *bitmaps, int64_t cap, int64_t *nnz_out, void *workspace,
                                   size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Visit schedule: an optional, derived re-packing of a layout for the attention kernel.
 *
 * A mask that keeps a band next to the diagonal (the constant context window that the figure of
 * Section 5.1 shows for self-attention) plus scattered isolated connections has a kept entry in
 * nearly every tile of a long sequence, although few tiles hold many.  The schedule lists, per
 * block row, "entries" of 64 keys each: a stored tile whose visible part
 * spans at least `min_cols` distinct key columns stays a run of 64 consecutive keys; the visible
 * columns of all other tiles of the block row are packed into gathered entries of 64 arbitrary,
 * distinct keys (grouped by which 32-query groups of the block row use a column, so that most
 * gathered entries concern one group only; the order inside an entry carries no meaning).  The causal limit (if any) is folded into the entry bitmaps, so a schedule must
 * be used with the same `causal` flag and the same layout it was built from.  It is a pure
 * function of its inputs (fixed order, no atomics) and never changes which (query, key) pairs
 * are evaluated -- only how they are grouped.
 *
 * Entry e of block row r is element row_ptr[r] + e of the arrays below; a block row never has
 * more entries than stored tiles, so arrays sized for the layout's `cap` always suffice.
 * ------------------------------------------------------------------------------------------- */
typedef struct ap_schedule {
    int32_t *cnt;      /* device int32 [H*nQB]        number of entries of each block row           */
    int32_t *start;    /* device int32 [cap]          >= 0: first key of 64 consecutive keys;
                                                      -1: gathered entry, keys listed in cols       */
    int32_t *cols;     /* device int32 [cap*64]       key index per slot of a gathered entry; empty
                                                      slots hold Lk                                 */
    uint64_t *bitmaps; /* device uint64 [cap*block_m] bit c of row rr: slot c of the entry is kept  */
} ap_schedule;

/*
 * Build the schedule of a layout (block_n must be 64, block_m 64 or 128).  `cap` is the number of
 * tiles the layout arrays and the schedule arrays have room for (>= the layout's nnz).
 * min_cols in [1, 65]: 1 keeps every tile as it is, 65 gathers everything; 0 selects the default.
 * All pointers inside `sched` (a host struct of device pointers) must be non-null and 8-byte
 * aligned for bitmaps, 4-byte for the rest.  Asynchronous on `stream`.
 */
ap_status ap_build_schedule(const int32_t *row_ptr, const int32_t *col_idx, const uint64_t *bitmaps,
                            int H, int Lq, int Lk, int block_m, int block_n, int64_t cap, int causal,
                            int min_cols, const ap_schedule *sched, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Masked attention forward (Section 3.2, masked-attention equation).
 *
 * For every batch b, head h and query i, over the keys j with mask[h,i,j] != 0 (and, if
 * `causal`, j <= i + (Lk - Lq): the auto-regressive mask composes with the pruning mask):
 *
 *     s_ij = scale * <Q[b,h,i,:], K[b,h,j,:]>
 *     lse[b,h,i] = ln sum_j exp(s_ij)
 *     O[b,h,i,:] = sum_j exp(s_ij - lse[b,h,i]) * V[b,h,j,:]
 *
 * A query with no visible kept key gets O = 0 and lse = -infinity.
 *
 *   Q, O          [B, H, Lq, D]; K, V  [B, H, Lk, D]; element type `dtype`; the last dimension
 *                 is contiguous; stride_x = {batch, head, sequence} strides in ELEMENTS (host
 *                 pointers to 3 int64).  Base pointers and row starts must be 16-byte aligned
 *                 (strides multiples of 8 elements for bf16, 4 for fp32).  O must not alias
 *                 Q, K or V.  Inputs must be finite: a pruned key's value row is still
 *                 multiplied by an exact zero inside a visited tile.
 *   lse           out, float [B, H, Lq] contiguous, or NULL
 *   row_ptr, col_idx, bitmaps   layout from ap_build_layout with the same H, Lq, Lk, block_m,
 *                 block_n; read-only, reusable across any number of calls
 *   sched         NULL, or a schedule built from this layout with the same `causal` (host
 *                 pointer to a struct of device pointers); bf16 only
 *   causal        nonzero = also hide future keys; requires Lk >= Lq
 *   softmax_scale <= 0 selects 1/sqrt(D)
 *
 * Supported: D in {32, 64, 128}; block_n = 64; block_m = 64 (both dtypes) or 128 (bf16); with a
 * schedule (here and in every call below that takes one), sequence lengths and row strides in
 * bytes below 2^24.  Returns AP_ERR_UNSUPPORTED otherwise.
 * ------------------------------------------------------------------------------------------- */
ap_status ap_sparse_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *lse,
                             ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                             const int64_t *stride_q, const int64_t *stride_k,
                             const int64_t *stride_v, const int64_t *stride_o,
                             const int32_t *row_ptr, const int32_t *col_idx,
                             const uint64_t *bitmaps, int block_m, int block_n,
                             const ap_schedule *sched, int causal, float softmax_scale,
                             void *stream);

/*
 * The same under the top-left Lq x Lk corner of a mask whose layout (and schedule) were built once
 * for Lq_layout x Lk_layout (Section 6: sequence lengths vary across a data set while the mask of
 * a layer and head is fixed): one layout serves every length, nothing is rebuilt per call.  The
 * result is that of ap_sparse_attn_fwd with the layout of the cropped mask (ap_build_layout_cropped).
 *
 *   Lq <= Lq_layout, Lk <= Lk_layout; Q, O have Lq rows, K, V have Lk rows
 *   causal        as in ap_sparse_attn_fwd, aligned to THIS call's sizes: j <= i + (Lk - Lq).  A
 *                 schedule has the limit of the layout's sizes folded in, so with `causal` and a
 *                 schedule Lk - Lq must equal Lk_layout - Lq_layout (e.g. self-attention cropped
 *                 to a shorter length), else AP_ERR_INVALID_ARG
 *   everything else as in ap_sparse_attn_fwd.  Supported: dtype = AP_BF16.
 */
ap_status ap_sparse_attn_fwd_cropped(const void *Q, const void *K, const void *V, void *O, float *lse,
                                     ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                     const int64_t *stride_q, const int64_t *stride_k,
                                     const int64_t *stride_v, const int64_t *stride_o,
                                     const int32_t *row_ptr, const int32_t *col_idx,
                                     const uint64_t *bitmaps, int block_m, int block_n, int Lq_layout,
                                     int Lk_layout, const ap_schedule *sched, int causal,
                                     float softmax_scale, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Masked attention forward for few queries against many keys (the Transformer-XL setting of
 * Section 4.1: a short segment attends to a long cached memory; the mask of such a layer is
 * Lq x Lk with Lk >> Lq and the causal limit is aligned bottom-right).
 *
 * Same arguments, same result (up to rounding) as ap_sparse_attn_fwd, but the tiles (or
 * schedule entries) of every block row are cut into `splits` contiguous chunks that run as
 * separate workgroups; each writes a normalised fp32 partial output and its log-sum-exp to the
 * workspace and a second kernel merges them:
 *     lse = ln sum_s exp(lse_s),   O = sum_s exp(lse_s - lse) O_s.
 * With one or two block rows per (batch, head) the ordinary call would use B*H*ceil(Lq/64)
 * workgroups; choose splits so that this number times splits reaches a few per compute unit.
 *
 *   splits        >= 1 (1 is allowed and only adds the merge), at most 1024
 *   workspace     device scratch of at least ap_fwd_split_workspace_bytes(B, H, Lq, D, splits)
 *                 bytes, 16-byte aligned
 *
 * Supported: dtype = AP_BF16, block_m = block_n = 64, D in {32, 64, 128}.  Deterministic.
 * ------------------------------------------------------------------------------------------- */
size_t ap_fwd_split_workspace_bytes(int B, int H, int Lq, int D, int splits);

ap_status ap_sparse_attn_fwd_split(const void *Q, const void *K, const void *V, void *O, float *lse,
                                   ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                   const int64_t *stride_q, const int64_t *stride_k,
                                   const int64_t *stride_v, const int64_t *stride_o,
                                   const int32_t *row_ptr, const int32_t *col_idx,
                                   const uint64_t *bitmaps, int block_m, int block_n,
                                   const ap_schedule *sched, int causal, float softmax_scale,
                                   int splits, void *workspace, size_t workspace_bytes,
                                   void *stream);

/*
 * ap_sparse_attn_fwd_split for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without the workspace, same kernels, same result bit for bit.  The partial outputs
 * live in a device array that is part of the library's code object (each GPU the library runs on
 * holds AP_FWD_SPLIT_STATIC_MAX_BYTES of it until the process ends); the call allocates and frees
 * nothing and calls no allocating routine.
 *
 *   - ap_fwd_split_workspace_bytes(B, H, Lq, D, splits) must not exceed
 *     AP_FWD_SPLIT_STATIC_MAX_BYTES, else AP_ERR_CAPACITY (checked on the host, before anything
 *     else happens).
 *   - The first call on a device looks up that device's copy of the array (one runtime query, no
 *     allocation); make that first call outside graph capture.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two
 *     streams, two host threads) race; serialise them.  Nothing in the array has to start at
 *     zero (every chunk writes its whole partial result before the merge reads it), so the call
 *     clears nothing and the previous call's contents are simply overwritten.
 */
#define AP_FWD_SPLIT_STATIC_MAX_BYTES ((size_t)32 << 20)

ap_status ap_sparse_attn_fwd_split_static(const void *Q, const void *K, const void *V, void *O, float *lse,
                                          ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                          const int64_t *stride_q, const int64_t *stride_k,
                                          const int64_t *stride_v, const int64_t *stride_o,
                                          const int32_t *row_ptr, const int32_t *col_idx,
                                          const uint64_t *bitmaps, int block_m, int block_n,
                                          const ap_schedule *sched, int causal, float softmax_scale,
                                          int splits, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Masked attention forward for one or a few queries against many keys (the limit of the
 * cached-memory setting of Section 4.1: a new position attends to everything stored before it under
 * the layer's fixed mask; with `causal` the limit is aligned bottom-right as everywhere else).
 *
 * Same arguments as ap_sparse_attn_fwd_split without the schedule, same result up to rounding as
 * ap_sparse_attn_fwd.  `splits` workgroups per (batch, head, query) read the K and V rows of that
 * query's kept keys and nothing else; the probabilities stay in fp32 (they are not rounded to bf16
 * before multiplying V).  Meant for Lq up to a few dozen; correct for any Lq.
 *
 *   splits        >= 1, at most 1024; 1 writes O directly and needs no workspace; choose it so
 *                 that B*H*Lq*splits reaches the number of compute units (256)
 *   workspace     for splits > 1: device scratch of at least
 *                 ap_fwd_split_workspace_bytes(B, H, Lq, D, splits) bytes, 16-byte aligned
 *
 * Supported: dtype = AP_BF16, D in {32, 64, 128}, block_n = 64, block_m = 64 or 128.
 * One launch, two with splits > 1.  Deterministic.
 * ------------------------------------------------------------------------------------------- */
ap_status ap_sparse_attn_decode(const void *Q, const void *K, const void *V, void *O, float *lse,
                                ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                const int64_t *stride_q, const int64_t *stride_k,
                                const int64_t *stride_v, const int64_t *stride_o,
                                const int32_t *row_ptr, const int32_t *col_idx,
                                const uint64_t *bitmaps, int block_m, int block_n, int causal,
                                float softmax_scale, int splits, void *workspace,
                                size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Masked attention forward with the 1.5-entmax normaliser (Section 6: the experiments are repeated
 * with 1.5-entmax in place of softmax, together with the pruning mask).
 *
 * For every batch b, head h and query i, over the keys j that ap_sparse_attn_fwd would use, with
 * x_ij = scale * <Q[b,h,i,:], K[b,h,j,:]> / 2:
 *
 *     p_ij = max(x_ij - tau[b,h,i], 0)^2 ,  tau[b,h,i] such that sum_j p_ij = 1
 *     O[b,h,i,:] = sum_j p_ij V[b,h,j,:]
 *
 * (the optimality conditions of 1.5-entmax; many p_ij are exactly 0).  tau is found by Newton's
 * iteration, which rises monotonically to the root: a row stops when |sum_j p_ij - 1| <= 1e-5 at
 * its tau, or after the one further step taken from a tau with |sum_j p_ij - 1| <= 1e-2 (the
 * steps converge quadratically, so the returned tau leaves |sum_j p_ij - 1| <= 1e-4).  O is
 * divided by the attained sum, so its weights sum to one whatever the residual; the backward call
 * forms p from the returned tau without that division.  A query with no visible kept key gets
 * O = 0 and tau = +infinity.
 *
 *   tau           out, float [B, H, Lq] contiguous, or NULL
 *   everything else as in ap_sparse_attn_fwd; a block row with more than 64 schedule entries
 *   walks the layout's tiles instead (same result)
 *
 * Supported: dtype = AP_BF16, block_m = block_n = 64, D in {32, 64, 128}.  One launch; the tiles of
 * a block row are swept several times (scores are recomputed, not stored).  Deterministic.
 * ------------------------------------------------------------------------------------------- */
ap_status ap_sparse_attn_entmax15_fwd(const void *Q, const void *K, const void *V, void *O, float *tau,
                                      ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                      const int64_t *stride_q, const int64_t *stride_k,
                                      const int64_t *stride_v, const int64_t *stride_o,
                                      const int32_t *row_ptr, const int32_t *col_idx,
                                      const uint64_t *bitmaps, int block_m, int block_n,
                                      const ap_schedule *sched, int causal, float softmax_scale,
                                      void *stream);

/* ---------------------------------------------------------------------------------------------
 * Backward pass of masked attention (Section 3.2, algorithm step 4: the pruned model F' is
 * trained, which needs the gradients of the masked-attention equation).
 *
 * With P_ij = exp(s_ij - lse_i) on kept, visible entries and 0 elsewhere (s and lse as in
 * ap_sparse_attn_fwd), and dP_ij = <dO[b,h,i,:], V[b,h,j,:]>:
 *
 *     dV[b,h,j,:] = sum_i P_ij dO[b,h,i,:]
 *     dS_ij       = P_ij (dP_ij - sum_d dO[b,h,i,d] O[b,h,i,d])
 *     dQ[b,h,i,:] = scale sum_j dS_ij K[b,h,j,:]        dK[b,h,j,:] = scale sum_i dS_ij Q[b,h,i,:]
 *
 * dK and dV are accumulated per block column of the layout, which needs the layout's transpose:
 *
 * ap_build_layout_transpose: for every (head, block column kb) the tiles of that column in
 * ascending block-row order.
 *   row_ptr, col_idx   from ap_build_layout (same H, Lq, Lk, block_m, block_n, cap)
 *   col_ptr       out, int32 [H * ceil(Lk/block_n) + 1]: tiles of column c are
 *                 [col_ptr[c], col_ptr[c+1])
 *   row_idx       out, int32 [cap]: block row qb of each of them
 *   tile_idx      out, int32 [cap]: its position in col_idx / bitmaps
 *   A truncated layout (more tiles than cap) must not be transposed.  Three launches, deterministic.
 *
 * ap_sparse_attn_bwd:
 *   Q, K, V, O, dO, lse   the forward call's inputs and outputs and the gradient of O; O and dO
 *                 share stride_o, dQ shares stride_q, dK stride_k, dV stride_v (all as in
 *                 ap_sparse_attn_fwd); lse float [B, H, Lq] contiguous (required)
 *   dQ, dK, dV    out; every element is written (zeros where nothing contributes); must not
 *                 alias any input
 *   workspace     device scratch of at least ap_bwd_workspace_bytes(B, H, Lq) bytes, 16-byte
 *                 aligned (the row sums of dO * O)
 *
 * Supported: dtype = AP_BF16, D in {32, 64, 128}, block_m = block_n = 64.  Three launches.
 * Deterministic (no floating-point atomics): dQ is formed per block row, dK and dV per block
 * column, each recomputing the scores of its tiles.
 * ------------------------------------------------------------------------------------------- */
ap_status ap_build_layout_transpose(const int32_t *row_ptr, const int32_t *col_idx, int H, int Lq,
                                    int Lk, int block_m, int block_n, int64_t cap, int32_t *col_ptr,
                                    int32_t *row_idx, int32_t *tile_idx, void *stream);

size_t ap_bwd_workspace_bytes(int B, int H, int Lq);

ap_status ap_sparse_attn_bwd(const void *Q, const void *K, const void *V, const void *O,
                             const void *dO, const float *lse, void *dQ, void *dK, void *dV,
                             ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                             const int64_t *stride_q, const int64_t *stride_k,
                             const int64_t *stride_v, const int64_t *stride_o,
                             const int32_t *row_ptr, const int32_t *col_idx,
                             const uint64_t *bitmaps, const int32_t *col_ptr,
                             const int32_t *row_idx, const int32_t *tile_idx, int block_m,
                             int block_n, int causal, float softmax_scale, void *workspace,
                             size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Backward pass over visit schedules: the same gradients as ap_sparse_attn_bwd (same passage of
 * the paper), skipping what the scheduled forward pass skips.
 *
 * dQ walks the row schedule of ap_build_schedule (entries of 64 consecutive or 64 gathered keys
 * per block row).  dK and dV walk a column schedule, the same structure with rows and columns
 * swapped, built from the transposed layout by ap_build_col_schedule: entry e of block column c
 * is element col_ptr[c] + e of its arrays;
 *     cnt   [2 * H * nKB + H], nKB = ceil(Lk/64): the entries of each block column [H * nKB],
 *                              then the visiting order of each head's block columns [H * nKB]
 *                              (columns with at least twice the head's mean number of entries
 *                              first), then the number of such columns per head [H]
 *     start [cap]              >= 0: first query of 64 consecutive queries; -1: gathered queries
 *     cols  [cap*64]           query index per slot of a gathered entry; empty slots hold Lq
 *     bitmaps [cap*64]         per query slot: bit c set = key 64*kb + c kept and visible
 * A stored tile in which at least min_rows query rows hold a visible kept entry stays one entry of
 * consecutive queries; the rows of the other tiles that hold one are packed, in ascending order,
 * into gathered entries.  min_rows in [1, 65]: 1 keeps every tile with a visible entry as it is,
 * 65 gathers everything; 0 selects the default.  Tiles without a visible kept entry are dropped.
 *
 * ap_sparse_attn_bwd_sched takes the arguments of ap_sparse_attn_bwd plus
 *   sched         NULL (dQ walks the layout's tiles), or the row schedule built from this layout
 *                 with the same `causal`
 *   col_sched     NULL (dK, dV walk the transposed layout), or the column schedule built from
 *                 this layout's transpose with the same `causal`
 * Same support, same determinism; results differ from ap_sparse_attn_bwd only by the order of
 * the fp32 sums.
 * ------------------------------------------------------------------------------------------- */
ap_status ap_build_col_schedule(const int32_t *col_ptr, const int32_t *row_idx, const int32_t *tile_idx,
                                const uint64_t *bitmaps, int H, int Lq, int Lk, int block_m,
                                int block_n, int64_t cap, int causal, int min_rows,
                                const ap_schedule *col_sched, void *stream);

ap_status ap_sparse_attn_bwd_sched(const void *Q, const void *K, const void *V, const void *O,
                                   const void *dO, const float *lse, void *dQ, void *dK, void *dV,
                                   ap_dtype dtype, int B, int H, int Lq, int Lk, int D,
                                   const int64_t *stride_q, const int64_t *stride_k,
                                   const int64_t *stride_v, const int64_t *stride_o,
                                   const int32_t *row_ptr, const int32_t *col_idx,
                                   const uint64_t *bitmaps, const int32_t *col_ptr,
                                   const int32_t *row_idx, const int32_t *tile_idx, int block_m,
                                   int block_n, const ap_schedule *sched,
                                   const ap_schedule *col_sched, int causal, float softmax_scale,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Backward pass of ap_sparse_attn_entmax15_fwd (Section 6: the models there are trained with the
 * 1.5-entmax normaliser under the pruning mask).
 *
 * With x_ij, tau and p_ij as in ap_sparse_attn_entmax15_fwd, u_ij = max(x_ij - tau_i, 0) (so
 * p_ij = u_ij^2) and g_ij = <dO[b,h,i,:], V[b,h,j,:]>, holding sum_j p_ij = 1 fixed:
 *
 *     gbar_i      = sum_j u_ij g_ij / sum_j u_ij
 *     dS_ij       = u_ij (g_ij - gbar_i)                 (gradient with respect to scale * <Q_i, K_j>)
 *     dV[b,h,j,:] = sum_i p_ij dO[b,h,i,:]
 *     dQ[b,h,i,:] = scale sum_j dS_ij K[b,h,j,:]         dK[b,h,j,:] = scale sum_i dS_ij Q[b,h,i,:]
 *
 *   Q, K, V, dO   as in ap_sparse_attn_bwd (dO uses stride_o); O is not needed
 *   tau           float [B, H, Lq] contiguous, the forward call's output (required)
 *   sched, col_sched   the row schedule and the column schedule of the layout (both required,
 *                 built with the same `causal`)
 *   workspace     device scratch of at least ap_entmax15_bwd_workspace_bytes(B, H, Lq) bytes,
 *                 16-byte aligned (gbar)
 *   everything else as in ap_sparse_attn_bwd_sched
 *
 * Supported: dtype = AP_BF16, D in {32, 64, 128}, block_m = block_n = 64.  Three launches (gbar,
 * dQ, dK/dV).  Deterministic.
 * ------------------------------------------------------------------------------------------- */
size_t ap_entmax15_bwd_workspace_bytes(int B, int H, int Lq);

ap_status ap_sparse_attn_entmax15_bwd(const void *Q, const void *K, const void *V, const void *dO,
                                      const float *tau, void *dQ, void *dK, void *dV, ap_dtype dtype,
                                      int B, int H, int Lq, int Lk, int D, const int64_t *stride_q,
                                      const int64_t *stride_k, const int64_t *stride_v,
                                      const int64_t *stride_o, const int32_t *row_ptr,
                                      const int32_t *col_idx, const uint64_t *bitmaps,
                                      const int32_t *col_ptr, const int32_t *row_idx,
                                      const int32_t *tile_idx, int block_m, int block_n,
                                      const ap_schedule *sched, const ap_schedule *col_sched, int causal,
                                      float softmax_scale, void *workspace, size_t workspace_bytes,
                                      void *stream);

/* ---------------------------------------------------------------------------------------------
 * Mask construction, step 1: accumulate attention matrices into the mean map (Section 3.2,
 * Eq. (1)).
 *
 * For every head h, query i and key j (if `causal`, only j <= i + (Lk - Lq)):
 *
 *     abar[h,i,j] += weight * sum_b  exp(s_bij) / sum_j' exp(s_bij'),   s_bij = scale * <Q[b,h,i,:], K[b,h,j,:]>
 *
 * i.e. the attention matrices A_b = softmax(Q_b K_b^T / sqrt(d_k)) of the B examples of this call
 * (Section 3.2: the masked-attention equation with the zero mask), summed element-wise.  Zero
 * `abar`, then call once per batch of the data set with weight = 1/n (n = number of examples
 * in the whole set) to obtain Eq. (1)'s mean; the running sum is kept in fp32.  Entries that
 * causality hides are neither read nor written.
 *
 *   Q [B, H, Lq, D], K [B, H, Lk, D]   as in ap_sparse_attn_fwd (bf16 only)
 *   abar          in/out, float [H, Lq, Lk] contiguous
 *   workspace     device scratch of at least ap_attention_maps_workspace_bytes(B, H, Lq) bytes
 *                 (the row-wise log-sum-exp of the scores), 16-byte aligned; contents undefined
 *                 before and after
 *
 * Supported: dtype = AP_BF16, D in {32, 64, 128}.  Two launches on `stream`.  Deterministic.
 * ------------------------------------------------------------------------------------------- */
size_t ap_attention_maps_workspace_bytes(int B, int H, int Lq);

ap_status ap_accumulate_attention_maps(const void *Q, const void *K, ap_dtype dtype, int B, int H,
                                       int Lq, int Lk, int D, const int64_t *stride_q,
                                       const int64_t *stride_k, int causal, float softmax_scale,
                                       float weight, float *abar, void *workspace,
                                       size_t workspace_bytes, void *stream);

/* The same when the model's own attention call has already run on these Q and K: `lse` is the
 * log-sum-exp [B, H, Lq] that ap_sparse_attn_fwd returns for the all-ones mask with the same
 * `causal` and scale (the unpruned model of step 2 of Section 3.2's procedure computes it anyway).
 * The pass that would recompute the row statistics is skipped: one small launch and the
 * accumulation.  Everything else as above, workspace included. */
ap_status ap_accumulate_attention_maps_lse(const void *Q, const void *K, const float *lse, ap_dtype dtype,
                                           int B, int H, int Lq, int Lk, int D, const int64_t *stride_q,
                                           const int64_t *stride_k, int causal, float softmax_scale,
                                           float weight, float *abar, void *workspace,
                                           size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Mask construction, step 2: layer-wise percentile threshold and pruning mask (Section 3.2,
 * paragraph before Eq. (2), and Eq. (2)).
 *
 * `abar` holds the mean maps of ALL heads of one attention layer.  With its N participating
 * entries (all H*Lq*Lk of them, or, if `causal`, those with j <= i + (Lk - Lq)) in ascending
 * order v[0] <= ... <= v[N-1], the threshold is the order statistic
 *
 *     tau = v[ floor(prune_fraction * N) ]          (no interpolation; +infinity if the rank is N)
 *
 * and an entry is pruned iff abar[h,i,j] < tau (strict: ties with tau are kept), so that with
 * distinct values exactly floor(prune_fraction * N) entries are pruned.  Output is the keep
 * mask that ap_build_layout consumes: mask[h,i,j] = 1 if participating and abar[h,i,j] >= tau,
 * else 0.  The rank is computed in double precision on the host exactly as written above.
 *
 *   abar          float [H, Lq, Lk] contiguous, 16-byte aligned; values must be >= 0 and not
 *                 NaN (they are means of probabilities)
 *   prune_fraction  p of the paper as a fraction, 0 <= p <= 1
 *   mask          out, uint8 [H, Lq, Lk] contiguous; or NULL to compute the threshold only (then
 *                 tau_out is required; ap_build_layout_from_map takes it from there)
 *   tau_out       out, one float (device), or NULL
 *   workspace     device scratch of at least ap_prune_mask_workspace_bytes() bytes, 16-byte
 *                 aligned; contents undefined before and after
 *
 * Exact: tau is an element of abar, found by radix selection over the bit patterns in two sweeps
 * over the map (a histogram of the leading key bits, then the candidates of the selected interval;
 * more histogram levels only when that interval holds a very large number of ties); integer
 * atomics only, so the result is bit-identical from run to run.
 * ------------------------------------------------------------------------------------------- */
size_t ap_prune_mask_workspace_bytes(void);

ap_status ap_prune_mask(const float *abar, int H, int Lq, int Lk, int causal, double prune_fraction,
                        uint8_t *mask, float *tau_out, void *workspace, size_t workspace_bytes,
                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AP_H */
