/* CPU oracle (test infrastructure only): the gated decay recurrence of Sec. 2.1,
 * Eq. 1, stepped token by token exactly as the equation is written. */
#include "ratsparse_ref.h"

void ref_rat_scan(int64_t BH, int64_t T, int64_t D, const float *k, const float *v,
                  const float *g, double *state_k, double *state_v, double *k_out,
                  double *v_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        double *sk = state_k + bh * D; /* k~_{t-1} */
        double *sv = state_v + bh * D; /* v~_{t-1} */
        for (int64_t t = 0; t < T; ++t) {
            const int64_t row = (bh * T + t) * D;
            for (int64_t c = 0; c < D; ++c) {
                const double gt = (double)g[row + c];
                sk[c] = gt * sk[c] + (1.0 - gt) * (double)k[row + c];
                sv[c] = gt * sv[c] + (1.0 - gt) * (double)v[row + c];
                k_out[row + c] = sk[c];
                v_out[row + c] = sv[c];
            }
        }
    }
}
