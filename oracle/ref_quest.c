/* CPU oracle (test infrastructure only): Quest block representatives, the page
 * score and the page selection of Eq. 3 (App. A.1, Quest paragraph). */
#include "ratsparse_ref.h"

#include <stdlib.h>
#include <string.h>

void ref_quest_page_meta(int64_t BH, int64_t Tcap, int64_t D, int64_t P,
                         const float *k_cache, int64_t T_valid, float *meta)
{
    const int64_t Np_cap = Tcap / P;
    const int64_t Np = (T_valid + P - 1) / P;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        for (int64_t p = 0; p < Np; ++p) {
            float *mn = meta + ((bh * Np_cap + p) * 2 + 0) * D;
            float *mx = meta + ((bh * Np_cap + p) * 2 + 1) * D;
            const int64_t t0 = p * P;
            const int64_t t1 = (t0 + P < T_valid) ? t0 + P : T_valid;
            for (int64_t c = 0; c < D; ++c) {
                float lo = k_cache[(bh * Tcap + t0) * D + c];
                float hi = lo;
                for (int64_t t = t0 + 1; t < t1; ++t) {
                    const float x = k_cache[(bh * Tcap + t) * D + c];
                    if (x < lo)
                        lo = x;
                    if (x > hi)
                        hi = x;
                }
                mn[c] = lo;
                mx[c] = hi;
            }
        }
    }
}

void ref_quest_scores(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t Np_cap,
                      const float *q, const float *meta, int64_t Np, double *scores)
{
    const int64_t G = Hq / Hkv;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < B * Hq; ++bh) {
        const int64_t b = bh / Hq, h = bh % Hq, kvh = h / G;
        const float *qv = q + bh * D;
        for (int64_t p = 0; p < Np; ++p) {
            const float *mn = meta + (((b * Hkv + kvh) * Np_cap + p) * 2 + 0) * D;
            const float *mx = mn + D;
            double s = 0.0;
            for (int64_t c = 0; c < D; ++c) {
                const double a = (double)qv[c] * (double)mn[c];
                const double z = (double)qv[c] * (double)mx[c];
                s += (a > z) ? a : z;
            }
            scores[bh * Np + p] = s;
        }
    }
}

void ref_quest_select(int64_t BHq, int64_t Np, const double *scores, int64_t K,
                      int64_t n_first, int64_t n_local, int32_t *idx)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < BHq; ++r) {
        uint8_t *forced = (uint8_t *)calloc((size_t)Np, 1);
        for (int64_t p = 0; p < Np; ++p)
            if (p < n_first || p >= Np - n_local)
                forced[p] = 1;
        ref_topk_row(Np, scores + r * Np, forced, K, idx + r * K);
        free(forced);
    }
}
