/* CPU oracle (test infrastructure only): MoBA routing at prefill (App. A.1, MoBA
 * paragraph): mean-pooled block representatives, per-query gate scores, Eq. 3. */
#include "ratsparse_ref.h"

#include <math.h>
#include <stdlib.h>

void ref_moba_block_means(int64_t BH, int64_t T, int64_t Tcap, int64_t D, int64_t block,
                          const float *k_cache, double *means)
{
    const int64_t Nb = (T + block - 1) / block;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        for (int64_t j = 0; j < Nb; ++j) {
            const int64_t t0 = j * block;
            const int64_t t1 = (t0 + block < T) ? t0 + block : T;
            for (int64_t c = 0; c < D; ++c) {
                double s = 0.0;
                for (int64_t t = t0; t < t1; ++t)
                    s += (double)k_cache[(bh * Tcap + t) * D + c];
                means[(bh * Nb + j) * D + c] = s / (double)(t1 - t0);
            }
        }
    }
}

void ref_moba_select(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t T,
                     int64_t block, int64_t K, int64_t n_first, const float *q,
                     const double *means, int64_t t_begin, int64_t t_end, int32_t *idx,
                     double *scores)
{
    const int64_t G = Hq / Hkv;
    const int64_t Nb = (T + block - 1) / block;
    const int64_t rows = t_end - t_begin;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < B * Hq; ++bh) {
        const int64_t b = bh / Hq, h = bh % Hq, kvh = h / G;
        double *s = (double *)malloc((size_t)Nb * sizeof(double));
        uint8_t *forced = (uint8_t *)malloc((size_t)Nb);
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t t = t_begin + r;
            const int64_t own = t / block; /* the block that holds the query itself */
            const float *qv = q + (bh * T + t) * D;
            /* candidates: own block (kept) and every block strictly before it */
            for (int64_t j = 0; j <= own; ++j) {
                const double *m = means + ((b * Hkv + kvh) * Nb + j) * D;
                double d = 0.0;
                for (int64_t c = 0; c < D; ++c)
                    d += (double)qv[c] * m[c];
                s[j] = d;
                forced[j] = (j == own || j < n_first) ? 1 : 0;
            }
            const int64_t avail = own + 1;
            const int64_t take = (K < avail) ? K : avail;
            int32_t *row_idx = idx + (bh * rows + r) * K;
            ref_topk_row(avail, s, forced, take, row_idx);
            for (int64_t j = take; j < K; ++j)
                row_idx[j] = -1;
            if (scores) {
                double *srow = scores + (bh * rows + r) * Nb;
                for (int64_t j = 0; j < Nb; ++j)
                    srow[j] = (j < own) ? s[j] : NAN;
            }
        }
        free(s);
        free(forced);
    }
}
