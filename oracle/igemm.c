/* CPU oracle, integer GEMM -- TEST INFRASTRUCTURE, never linked by the product.
 *
 * The quantized linear layer multiplies integer activation codes by integer
 * weight codes and accumulates in integers (the paper's W8A8 / W4A8 integer
 * arithmetic, Y = XW with one weight row per output channel).  This file is
 * that definition written out: a triple loop, 64-bit accumulation, and a check
 * that every sum fits the 32-bit accumulator the method uses.
 *
 * Threads split rows only (rows are independent); no blocking, no intrinsics.
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC
 */
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* acc[m,n] = sum_k xq[m,k] * wq[n,k].  xq [M,K], wq [N,K], acc [M,N], row-major.
 * Returns the number of sums that do not fit int32 (0 = all exact). */
int64_t oracle_igemm(const int8_t *xq, const int8_t *wq, int M, int N, int K, int32_t *acc)
{
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int k = 0; k < K; ++k)
                s += (int64_t)xq[(size_t)m * K + k] * (int64_t)wq[(size_t)n * K + k];
            if (s > INT32_MAX || s < INT32_MIN)
                ++bad;
            acc[(size_t)m * N + n] = (int32_t)s;
        }
    }
    return bad;
}

/* Group-wise variant for W4A8: for every group g of `group` consecutive k,
 *   part[m,g,n] = sum_{k in g} xq[m,k] * q[n,k]          (exact integer)
 *   accf[m,n]   = sum_g (double)part[m,g,n] * sw[n,g]     (fp64, g ascending)
 *   total[m,n]  = sum_g part[m,g,n]                       (exact integer)
 * q [N,K] holds the sign-extended int4 codes, sw [N,K/group] the group scales
 * widened to double.  `part` may be NULL.  Returns the number of overflows. */
int64_t oracle_igemm_grouped(const int8_t *xq, const int8_t *q, const double *sw,
                             int M, int N, int K, int group,
                             double *accf, int32_t *total, int32_t *part)
{
    const int G = K / group;
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double f = 0.0;
            int64_t t = 0;
            for (int g = 0; g < G; ++g) {
                int64_t s = 0;
                for (int k = g * group; k < (g + 1) * group; ++k)
                    s += (int64_t)xq[(size_t)m * K + k] * (int64_t)q[(size_t)n * K + k];
                if (s > INT32_MAX || s < INT32_MIN)
                    ++bad;
                if (part)
                    part[((size_t)m * G + g) * N + n] = (int32_t)s;
                f += (double)s * sw[(size_t)n * G + g];
                t += s;
            }
            if (t > INT32_MAX || t < INT32_MIN)
                ++bad;
            accf[(size_t)m * N + n] = f;
            total[(size_t)m * N + n] = (int32_t)t;
        }
    }
    return bad;
}
