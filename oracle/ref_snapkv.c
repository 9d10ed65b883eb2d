/* CPU oracle (test infrastructure only): SnapKV cache compression (App. A.1, SnapKV
 * paragraph): observation-window attention votes, pooling, Eq. 3 over single
 * tokens, and the gather of the retained entries. */
#include "ratsparse_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

void ref_snapkv_votes(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t T,
                      int64_t Tcap, int64_t W, const float *q_win, const float *k_cache,
                      double scale, double *votes, double *window_mass)
{
    const int64_t G = Hq / Hkv;
    const int64_t L = T - W; /* prefix positions that can be voted on */
#pragma omp parallel for schedule(static)
    for (int64_t bk = 0; bk < B * Hkv; ++bk) {
        const int64_t b = bk / Hkv, kvh = bk % Hkv;
        const float *kb = k_cache + bk * Tcap * D;
        double *vote = votes + bk * L;
        for (int64_t i = 0; i < L; ++i)
            vote[i] = 0.0;
        double *logit = (double *)malloc((size_t)T * sizeof(double));
        for (int64_t hg = 0; hg < G; ++hg) {
            const int64_t h = kvh * G + hg;
            for (int64_t w = 0; w < W; ++w) {
                const int64_t pos = L + w; /* absolute position of this query */
                const float *qv = q_win + ((b * Hq + h) * W + w) * D;
                double top = -INFINITY;
                for (int64_t i = 0; i <= pos; ++i) {
                    double s = 0.0;
                    for (int64_t c = 0; c < D; ++c)
                        s += (double)qv[c] * (double)kb[i * D + c];
                    logit[i] = scale * s;
                    if (logit[i] > top)
                        top = logit[i];
                }
                double denom = 0.0;
                for (int64_t i = 0; i <= pos; ++i)
                    denom += exp(logit[i] - top);
                for (int64_t i = 0; i < L; ++i)
                    vote[i] += exp(logit[i] - top) / denom;
                if (window_mass) {
                    double m = 0.0;
                    for (int64_t i = L; i <= pos; ++i)
                        m += exp(logit[i] - top) / denom;
                    window_mass[(b * Hq + h) * W + w] = m;
                }
            }
        }
        free(logit);
    }
}

void ref_maxpool1d(int64_t rows, int64_t L, int64_t kernel, const double *in, double *out)
{
    const int64_t half = kernel / 2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t i = 0; i < L; ++i) {
            const int64_t lo = (i - half < 0) ? 0 : i - half;
            const int64_t hi = (i + half > L - 1) ? L - 1 : i + half;
            double m = in[r * L + lo];
            for (int64_t j = lo + 1; j <= hi; ++j)
                if (in[r * L + j] > m)
                    m = in[r * L + j];
            out[r * L + i] = m;
        }
    }
}

void ref_snapkv_select_gather(int64_t BH, int64_t T, int64_t Tcap, int64_t D, int64_t W,
                              int64_t K_keep, const double *pooled, const float *k_cache,
                              const float *v_cache, int64_t Tcap_out, int32_t *idx,
                              float *kc_out, float *vc_out)
{
    const int64_t L = T - W;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        int32_t *sel = idx + bh * K_keep;
        ref_topk_row(L, pooled + bh * L, 0, K_keep, sel);
        for (int64_t j = 0; j < K_keep + W; ++j) {
            const int64_t src = (j < K_keep) ? sel[j] : L + (j - K_keep);
            memcpy(kc_out + (bh * Tcap_out + j) * D, k_cache + (bh * Tcap + src) * D,
                   (size_t)D * sizeof(float));
            memcpy(vc_out + (bh * Tcap_out + j) * D, v_cache + (bh * Tcap + src) * D,
                   (size_t)D * sizeof(float));
        }
    }
}
