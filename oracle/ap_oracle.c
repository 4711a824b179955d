/*
 * ap_oracle.c -- plain fp64 CPU oracle for Attention Pruning's masked attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct reference
 * that the GPU library is checked against.  It shares no code, header, table or
 * helper with the GPU path, and the product never calls it.
 *
 * What it computes (paper, Section 3.1 "Scaled Dot-Product Attention" and
 * Section 3.2, the masked-attention equation that follows Eq. (2)):
 *
 *     A~ = softmax( (Q K^T + M_p) / sqrt(d_k) ) V
 *
 * with M_p = 0 on kept connections and -infinity on pruned ones (Eq. (2) read
 * as an additive mask; its footnote says it is implemented by adding a large
 * negative value before the softmax).  -infinity entries contribute exp(.) = 0,
 * so the softmax runs over the kept keys only.  The mask carries no batch
 * index: it is one global pattern per head (Section 3.2, "global sparseness").
 * An auto-regressive model additionally hides future keys (caption of the
 * Transformer-XL figure: the pruning mask composes with the causal one); with
 * more keys than queries the causal diagonal is aligned to the bottom-right
 * corner, i.e. key j is visible to query i iff j <= i + (Lk - Lq).
 *
 * Readings taken where the paper is silent:
 *   - a query with no visible kept key gets O = 0 and lse = -infinity;
 *   - scale <= 0 selects the paper's 1/sqrt(d_k).
 *
 * Everything is plain loops in double precision; the softmax uses the two-pass
 * max-subtracted form, which equals the definition up to rounding.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the loops below will use (reported by the benchmark). */
int ap_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Masked softmax attention, Section 3.2 (equation after Eq. (2)).
 *
 *   Q    [B, H, Lq, D ]  contiguous, double
 *   K    [B, H, Lk, D ]
 *   V    [B, H, Lk, Dv]
 *   mask [H, Lq, Lk]     bytes, nonzero = connection kept (M_p = 0), zero = pruned (M_p = -inf)
 *   O    [B, H, Lq, Dv]  out
 *   lse  [B, H, Lq]      out, may be NULL: ln sum_{j kept} exp(s_ij)
 *
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int ap_oracle_masked_attention(const double *Q, const double *K, const double *V,
                               const uint8_t *mask,
                               int B, int H, int Lq, int Lk, int D, int Dv,
                               int causal, double scale,
                               double *O, double *lse)
{
    if (!Q || !K || !V || !mask || !O) return -1;
    if (B <= 0 || H <= 0 || Lq <= 0 || Lk <= 0 || D <= 0 || Dv <= 0) return -1;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);

    int failed = 0;
    const long long rows = (long long)B * H * Lq;

#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)Lk * sizeof(double));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 16)
        for (long long r = 0; r < rows; ++r) {
            if (!s) continue;
            const int i = (int)(r % Lq);
            const int h = (int)((r / Lq) % H);
            const int b = (int)(r / ((long long)Lq * H));

            const double *q = Q + (((size_t)b * H + h) * Lq + i) * D;
            const double *Kbh = K + ((size_t)b * H + h) * (size_t)Lk * D;
            const double *Vbh = V + ((size_t)b * H + h) * (size_t)Lk * Dv;
            const uint8_t *mrow = mask + ((size_t)h * Lq + i) * (size_t)Lk;
            double *o = O + (((size_t)b * H + h) * Lq + i) * Dv;

            /* last key the causal mask lets query i see */
            const long long jmax = causal ? (long long)i + ((long long)Lk - Lq) : (long long)Lk - 1;

            /* pass 1: scaled scores of the kept, visible keys and their maximum */
            double m = -INFINITY;
            int any = 0;
            for (int j = 0; j < Lk; ++j) {
                const int kept = (mrow[j] != 0) && ((long long)j <= jmax);
                if (!kept) continue;
                const double *k = Kbh + (size_t)j * D;
                double dot = 0.0;
                for (int t = 0; t < D; ++t) dot += q[t] * k[t];
                s[j] = dot * scale;
                if (!any || s[j] > m) m = s[j];
                any = 1;
            }

            for (int t = 0; t < Dv; ++t) o[t] = 0.0;
            if (!any) {
                if (lse) lse[r] = -INFINITY;
                continue;
            }

            /* pass 2: softmax denominator over the kept keys */
            double l = 0.0;
            for (int j = 0; j < Lk; ++j) {
                const int kept = (mrow[j] != 0) && ((long long)j <= jmax);
                if (kept) l += exp(s[j] - m);
            }
            if (lse) lse[r] = m + log(l);

            /* pass 3: probability-weighted sum of value rows */
            for (int j = 0; j < Lk; ++j) {
                const int kept = (mrow[j] != 0) && ((long long)j <= jmax);
                if (!kept) continue;
                const double p = exp(s[j] - m) / l;
                const double *v = Vbh + (size_t)j * Dv;
                for (int t = 0; t < Dv; ++t) o[t] += p * v[t];
            }
        }
        free(s);
    }
    return failed ? -1 : 0;
}

/*
 * Block-sparse layout of an element mask (Section 9.2 uses block-structured
 * sparseness patterns with a block size; here every block also keeps its
 * element bitmap so the element mask of Eq. (2) stays exact).
 *
 * Tiles are BM x BN windows of the [Lq, Lk] mask of one head, clipped at the
 * edges.  A tile exists iff any byte in its window is nonzero.  Block rows are
 * numbered r = h * nQB + qb with nQB = ceil(Lq / BM); inside a block row tiles
 * are listed by ascending block column kb.
 *
 *   row_ptr [H*nQB + 1]   exclusive prefix sum of tiles per block row
 *   col_idx [nnz]         kb of each tile                     (may be NULL)
 *   bitmaps [nnz*BM*W]    W = ceil(BN / 64) words per tile row (may be NULL):
 *                         bit (c % 64) of word c / 64 of local row rr of tile t
 *                         is mask[h, qb*BM + rr, kb*BN + c] != 0; positions
 *                         outside the mask are 0
 *
 * Returns the number of tiles (nnz).  Entries at positions >= cap are counted
 * but not written.  Returns -1 on bad arguments.
 */
long long ap_oracle_build_layout(const uint8_t *mask, int H, int Lq, int Lk, int BM, int BN,
                                 int32_t *row_ptr, int32_t *col_idx, uint64_t *bitmaps,
                                 long long cap)
{
    if (!mask || !row_ptr || H <= 0 || Lq <= 0 || Lk <= 0 || BM <= 0 || BN <= 0) return -1;
    const int nQB = (Lq + BM - 1) / BM;
    const int nKB = (Lk + BN - 1) / BN;
    const int W = (BN + 63) / 64;

    long long nnz = 0;
    for (int h = 0; h < H; ++h) {
        for (int qb = 0; qb < nQB; ++qb) {
            row_ptr[(size_t)h * nQB + qb] = (int32_t)nnz;
            for (int kb = 0; kb < nKB; ++kb) {
                /* does the window hold any kept entry? */
                int any = 0;
                for (int rr = 0; rr < BM && !any; ++rr) {
                    const int i = qb * BM + rr;
                    if (i >= Lq) break;
                    for (int c = 0; c < BN; ++c) {
                        const int j = kb * BN + c;
                        if (j >= Lk) break;
                        if (mask[((size_t)h * Lq + i) * Lk + j] != 0) { any = 1; break; }
                    }
                }
                if (!any) continue;
                if (nnz < cap) {
                    if (col_idx) col_idx[nnz] = kb;
                    if (bitmaps) {
                        for (int rr = 0; rr < BM; ++rr) {
                            for (int w = 0; w < W; ++w) {
                                uint64_t word = 0;
                                for (int bit = 0; bit < 64; ++bit) {
                                    const int c = w * 64 + bit;
                                    const int i = qb * BM + rr;
                                    const int j = kb * BN + c;
                                    if (c < BN && i < Lq && j < Lk &&
                                        mask[((size_t)h * Lq + i) * Lk + j] != 0)
                                        word |= (uint64_t)1 << bit;
                                }
                                bitmaps[((size_t)nnz * BM + rr) * W + w] = word;
                            }
                        }
                    }
                }
                ++nnz;
            }
        }
    }
    row_ptr[(size_t)H * nQB] = (int32_t)nnz;
    return nnz;
}
