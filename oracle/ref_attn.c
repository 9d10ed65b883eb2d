/* CPU oracle (test infrastructure only): sparse evaluation, Eq. 4, with f = softmax
 * over the selected tokens and logits multiplied by an explicit scale; the dense
 * path is the same with every token selected. */
#include "ratsparse_ref.h"

#include <math.h>
#include <stdlib.h>

/* softmax-weighted average of value rows over a list of token positions */
static void attend_tokens(int64_t D, const float *qv, const float *kbase, const float *vbase,
                          const int64_t *tok, int64_t n, double scale, double *out,
                          double *lse)
{
    double *logit = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    double top = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const float *kr = kbase + tok[j] * D;
        double s = 0.0;
        for (int64_t c = 0; c < D; ++c)
            s += (double)qv[c] * (double)kr[c];
        logit[j] = scale * s;
        if (logit[j] > top)
            top = logit[j];
    }
    for (int64_t c = 0; c < D; ++c)
        out[c] = 0.0;
    double denom = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        const double p = exp(logit[j] - top);
        denom += p;
        const float *vr = vbase + tok[j] * D;
        for (int64_t c = 0; c < D; ++c)
            out[c] += p * (double)vr[c];
    }
    if (n > 0)
        for (int64_t c = 0; c < D; ++c)
            out[c] /= denom;
    if (lse)
        *lse = (n > 0) ? top + log(denom) : -INFINITY;
    free(logit);
}

void ref_sparse_attn_decode(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t Tcap,
                            int64_t P, const float *q, const float *k_cache,
                            const float *v_cache, int64_t T_valid, double scale,
                            const int32_t *idx, int64_t K, double *out, double *lse)
{
    const int64_t G = Hq / Hkv;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < B * Hq; ++bh) {
        const int64_t b = bh / Hq, h = bh % Hq, kvh = h / G;
        const float *kb = k_cache + (b * Hkv + kvh) * Tcap * D;
        const float *vb = v_cache + (b * Hkv + kvh) * Tcap * D;
        int64_t cap = idx ? K * P : T_valid;
        int64_t *tok = (int64_t *)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(int64_t));
        int64_t n = 0;
        if (idx) {
            for (int64_t j = 0; j < K; ++j) {
                const int64_t p = idx[bh * K + j];
                if (p < 0)
                    continue;
                for (int64_t t = p * P; t < (p + 1) * P && t < T_valid; ++t)
                    tok[n++] = t;
            }
        } else {
            for (int64_t t = 0; t < T_valid; ++t)
                tok[n++] = t;
        }
        attend_tokens(D, q + bh * D, kb, vb, tok, n, scale, out + bh * D,
                      lse ? lse + bh : 0);
        free(tok);
    }
}

void ref_sparse_attn_prefill(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t T,
                             int64_t Tcap, int64_t block, const float *q,
                             const float *k_cache, const float *v_cache, double scale,
                             const int32_t *idx, int64_t K, int64_t t_begin,
                             int64_t t_end, double *out, double *lse)
{
    const int64_t G = Hq / Hkv;
    const int64_t rows = t_end - t_begin;
#pragma omp parallel for schedule(dynamic, 16) collapse(2)
    for (int64_t bh = 0; bh < B * Hq; ++bh) {
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t b = bh / Hq, h = bh % Hq, kvh = h / G;
            const int64_t t = t_begin + r;
            const float *kb = k_cache + (b * Hkv + kvh) * Tcap * D;
            const float *vb = v_cache + (b * Hkv + kvh) * Tcap * D;
            int64_t *tok = (int64_t *)malloc((size_t)(t + 1) * sizeof(int64_t));
            int64_t n = 0;
            if (idx) {
                for (int64_t j = 0; j < K; ++j) {
                    const int64_t blk = idx[(bh * rows + r) * K + j];
                    if (blk < 0)
                        continue;
                    for (int64_t i = blk * block; i < (blk + 1) * block && i <= t; ++i)
                        tok[n++] = i; /* causal: only positions i <= t */
                }
            } else {
                for (int64_t i = 0; i <= t; ++i)
                    tok[n++] = i;
            }
            attend_tokens(D, q + (bh * T + t) * D, kb, vb, tok, n, scale,
                          out + (bh * rows + r) * D, lse ? lse + bh * rows + r : 0);
            free(tok);
        }
    }
}
