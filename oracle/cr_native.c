/* CPU oracle, native part.  TEST INFRASTRUCTURE ONLY -- never linked into or
 * called by the product library.
 *
 * Plain C restatement of the per-segment partial gradient that every tree node
 * evaluates on its share of the data (Section III-A, CR.Execute step 1, with the
 * "b D" weighting notation of the same section), and of the full gradient of
 * eq. (3):
 *
 *     g[b,e) = sum_{j=b}^{e-1} x_j * (phi(x_j . w) - y_j)
 *
 * phi(z) = z (least squares) or the logistic function (targets in {0,1}).
 * X is row-major m x d, stored as fp32 or as bf16 bit patterns; every input is
 * widened exactly to fp64 and all arithmetic is fp64.  Rows are visited in
 * order; OpenMP splits the row range over threads, each with its own
 * accumulator, and the per-thread sums are added in thread order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { CRO_LINEAR = 0, CRO_LOGISTIC = 1 };
enum { CRO_F32 = 0, CRO_BF16 = 1 };

static double widen_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double logistic(double z)
{
    if (z >= 0.0)
        return 1.0 / (1.0 + exp(-z));
    double ez = exp(z);
    return ez / (1.0 + ez);
}

int cro_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* g_out[0..d) = sum over rows [row_begin,row_end) of x_j (phi(x_j.w) - y_j).  Returns 0, or -1 on bad arguments / allocation failure. */
int cro_segment_gradient(const void *X, int x_dtype, const float *y, const float *w,
                         int64_t d, int model, int64_t row_begin, int64_t row_end, double *g_out)
{
    if (!X || !y || !w || !g_out || d < 1 || row_end < row_begin)
        return -1;
    int nt = cro_num_threads();
    double *acc = calloc((size_t)nt * (size_t)d, sizeof(double));
    double *wd = malloc((size_t)d * sizeof(double));
    if (!acc || !wd) {
        free(acc);
        free(wd);
        return -1;
    }
    for (int64_t c = 0; c < d; ++c)
        wd[c] = (double)w[c];

#pragma omp parallel num_threads(nt)
    {
#ifdef _OPENMP
        int t = omp_get_thread_num();
#else
        int t = 0;
#endif
        double *g = acc + (size_t)t * (size_t)d;
        double *row = malloc((size_t)d * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t j = row_begin; j < row_end; ++j) {
            if (x_dtype == CRO_BF16) {
                const uint16_t *xr = (const uint16_t *)X + (size_t)j * (size_t)d;
                for (int64_t c = 0; c < d; ++c)
                    row[c] = widen_bf16(xr[c]);
            } else {
                const float *xr = (const float *)X + (size_t)j * (size_t)d;
                for (int64_t c = 0; c < d; ++c)
                    row[c] = (double)xr[c];
            }
            double z = 0.0;
            for (int64_t c = 0; c < d; ++c)
                z += row[c] * wd[c];
            double r = (model == CRO_LOGISTIC ? logistic(z) : z) - (double)y[j];
            for (int64_t c = 0; c < d; ++c)
                g[c] += r * row[c];
        }
        free(row);
    }
    for (int64_t c = 0; c < d; ++c) {
        double sum = 0.0;
        for (int t = 0; t < nt; ++t)
            sum += acc[(size_t)t * (size_t)d + (size_t)c];
        g_out[c] = sum;
    }
    free(acc);
    free(wd);
    return 0;
}

/* eq. (3): the whole data set is one segment. */
int cro_full_gradient(const void *X, int x_dtype, const float *y, const float *w,
                      int64_t m, int64_t d, int model, double *g_out)
{
    return cro_segment_gradient(X, x_dtype, y, w, d, model, 0, m, g_out);
}
