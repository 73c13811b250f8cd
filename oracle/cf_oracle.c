/*
 * CommFuse CPU oracle -- dense fp64 arithmetic (TEST INFRASTRUCTURE ONLY).
 *
 * This translation unit is the slow, plain, obviously-correct reference that
 * the HIP path is checked against.  It shares no code, header, table or
 * helper with the GPU library and nothing in the product path may link it.
 *
 * What it holds: the dense contraction that both collective definitions of
 * the paper reduce to (Sec. 3.1, "Common collective communications": a
 * reduce-scatter of row-parallel partial products, an all-gather followed by
 * a column-parallel product) and the element-wise sum of the data-parallel
 * gradient path (Sec. 3.1, Zero-DP paragraph).  Everything is a textbook
 * triple loop in IEEE double; there is no blocking, no reordering of the
 * k-sum and no vector intrinsics.  OpenMP only splits independent output
 * rows over threads.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* O[M x N] = A[M x K] * W[K x N], all row-major with explicit row strides.
 * The k-sum of every output element runs k = 0..K-1 in order. */
void cfo_gemm_f64(const double *A, int64_t lda, const double *W, int64_t ldw,
                  double *O, int64_t ldo, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *o = O + i * ldo;
        for (int64_t j = 0; j < N; ++j)
            o[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[i * lda + k];
            const double *w = W + k * ldw;
            for (int64_t j = 0; j < N; ++j)
                o[j] += a * w[j];
        }
    }
}

/* One output element by its definition: sum_k A[i][k] * W[k][j]. */
double cfo_dot_f64(const double *A, int64_t lda, const double *W, int64_t ldw,
                   int64_t i, int64_t j, int64_t K)
{
    double s = 0.0;
    for (int64_t k = 0; k < K; ++k)
        s += A[i * lda + k] * W[k * ldw + j];
    return s;
}

/* dst[e] = a[e] + b[e]  (the "B_in + O" of Alg. 2, element by element). */
void cfo_add_f64(const double *a, const double *b, double *dst, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e)
        dst[e] = a[e] + b[e];
}

int cfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
