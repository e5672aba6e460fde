/* CPU oracle, test infrastructure only: the plain definition of the layer's
 * accumulator  acc[m][o] = sum_k X[m][k] * W[o][k]   (Y = X . W^T, the goal
 * equation of Sec. 3.1), written as the triple loop it is.  int64 sums for INT8
 * operands, fp64 sums for operands already widened to double.  No blocking and
 * no reordering of the k sum; OpenMP only splits the independent (m, o) outputs.
 * Shares nothing with the HIP library. */
#include <stdint.h>

void oracle_gemm_i8_i64(const int8_t* X, const int8_t* W, int64_t M, int64_t O, int64_t K,
                        int64_t* acc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t o = 0; o < O; ++o) {
            const int8_t* x = X + m * K;
            const int8_t* w = W + o * K;
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int64_t)x[k] * (int64_t)w[k];
            acc[m * O + o] = s;
        }
}

void oracle_gemm_f64(const double* X, const double* W, int64_t M, int64_t O, int64_t K,
                     double* acc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t o = 0; o < O; ++o) {
            const double* x = X + m * K;
            const double* w = W + o * K;
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) s += x[k] * w[k];
            acc[m * O + o] = s;
        }
}

int oracle_omp_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
