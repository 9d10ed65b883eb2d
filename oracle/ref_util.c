/* CPU oracle (test infrastructure only): rounding to the cache dtype and the
 * generic top-K of Eq. 3.  Shares nothing with the HIP library. */
#include "ratsparse_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* number of OpenMP threads the following calls use (timing aid; no effect on results) */
void ref_set_num_threads(int n)
{
    if (n > 0) omp_set_num_threads(n);
}

/* bfloat16: 1 sign, 8 exponent, 7 stored mantissa bits => 8 significant bits, the
 * exponent range of float32.  A value x = m * 2^e with 0.5 <= |m| < 1 is rounded on
 * the grid 2^(e-8); below the smallest normal 2^-126 the grid is fixed at 2^-133.
 * rint() rounds halfway cases to even in the default rounding mode. */
static double round_one_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x))
        return x;
    int e;
    (void)frexp(x, &e);
    int grid = e - 8;
    if (grid < -133)
        grid = -133;
    double r = ldexp(rint(ldexp(x, -grid)), grid);
    /* largest finite bf16 is (2 - 2^-7) * 2^127; anything rounding past it is inf */
    const double big = ldexp(2.0 - ldexp(1.0, -7), 127);
    if (fabs(r) > big)
        r = (x > 0) ? INFINITY : -INFINITY;
    return r;
}

void ref_round_to_bf16(int64_t n, const double *x, float *y)
{
    for (int64_t i = 0; i < n; ++i)
        y[i] = (float)round_one_bf16(x[i]); /* exact: a bf16 value is a float */
}

typedef struct {
    double score;
    int forced;
    int32_t index;
} cand_t;

/* forced first, then score descending, then index ascending */
static int cand_before(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->forced != b->forced)
        return b->forced - a->forced;
    if (a->score > b->score)
        return -1;
    if (a->score < b->score)
        return 1;
    return (a->index > b->index) - (a->index < b->index);
}

static int int32_ascending(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

void ref_topk_row(int64_t M, const double *score, const uint8_t *forced, int64_t K,
                  int32_t *idx_out)
{
    if (K <= 0)
        return;
    cand_t *c = (cand_t *)malloc((size_t)M * sizeof(cand_t));
    for (int64_t i = 0; i < M; ++i) {
        c[i].score = score[i];
        c[i].forced = (forced && forced[i]) ? 1 : 0;
        c[i].index = (int32_t)i;
    }
    qsort(c, (size_t)M, sizeof(cand_t), cand_before);
    for (int64_t j = 0; j < K; ++j)
        idx_out[j] = c[j].index;
    qsort(idx_out, (size_t)K, sizeof(int32_t), int32_ascending);
    free(c);
}
