/*
 * CPU oracle for the LCMA GEMM path.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may link, load or call this file.  It is deliberately plain and
 * slow: no blocking, no fusion, no reordering beyond what the definitions say.
 *
 * What it holds
 *   oracle_gemm_f64 / oracle_gemm_i64
 *       C = A x B by the textbook definition (paper Eq. 1), C[i][j] = sum_p
 *       A[i][p]*B[p][j], summed in ascending p.  Loop order is i, p, j so the
 *       inner loop walks rows of B and C; every C[i][j] still receives its terms
 *       in ascending p, so the rounding order is that of the definition.
 *   oracle_lcma_f64 / oracle_lcma_i64
 *       The four-stage LCMA workflow (paper Sec. 2.1 Eq. 3-6, Algorithm 1):
 *       Combine A, Combine B, R block products, Combine H.  Intermediates are
 *       whole matrices in main memory exactly as Algorithm 1 describes.
 *   oracle_brent_residual
 *       Integer check that <m,k,n;R;U,V,W> is a matrix-multiplication scheme:
 *       substituting Eq. 3-5 into Eq. 6 and matching the coefficient of
 *       A_{i,a} B_{b,j} in C_{c,d} gives
 *          sum_r U[r,i,a] V[r,b,j] W[r,c,d] = [a==b][i==c][j==d].
 *
 * Conventions: row-major, leading dimensions in elements, U is R x m x k,
 * V is R x k x n, W is R x m x n (all row-major int32), block sizes M/m, K/k,
 * N/n must divide exactly (the reading taken for paper Sec. 2.1's ceilings).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
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

/* Eq. 1, fp64. */
void oracle_gemm_f64(int64_t M, int64_t N, int64_t K,
                     const double *A, int64_t lda,
                     const double *B, int64_t ldb,
                     double *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + i * ldc;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t p = 0; p < K; ++p) {
            const double a = A[i * lda + p];
            const double *b = B + p * ldb;
            for (int64_t j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

/* Eq. 1, exact integers. */
void oracle_gemm_i64(int64_t M, int64_t N, int64_t K,
                     const int64_t *A, int64_t lda,
                     const int64_t *B, int64_t ldb,
                     int64_t *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        int64_t *c = C + i * ldc;
        for (int64_t j = 0; j < N; ++j) c[j] = 0;
        for (int64_t p = 0; p < K; ++p) {
            const int64_t a = A[i * lda + p];
            const int64_t *b = B + p * ldb;
            for (int64_t j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

/* Rows [row0,row0+rows) of C = A x B only (used to sample big problems). */
void oracle_gemm_rows_f64(int64_t row0, int64_t rows, int64_t N, int64_t K,
                          const double *A, int64_t lda,
                          const double *B, int64_t ldb,
                          double *Crows, int64_t ldc)
{
    oracle_gemm_f64(rows, N, K, A + row0 * lda, lda, B, ldb, Crows, ldc);
}

/*
 * The LCMA workflow, written once for a value type T.
 *   Stage 1 (Eq. 3): At[r] = sum_{i,l} U[r,i,l] * A_{i,l}        (bm x bk)
 *   Stage 2 (Eq. 4): Bt[r] = sum_{l,j} V[r,l,j] * B_{l,j}        (bk x bn)
 *   Stage 3 (Eq. 5): H[r]  = At[r] x Bt[r]                        (bm x bn)
 *   Stage 4 (Eq. 6): C_{i,j} = sum_r W[r,i,j] * H[r]
 * Zero coefficients are skipped as in Algorithm 1; sums run in ascending index.
 * Returns 0, or 1 on a shape that does not divide, or 2 when out of memory.
 */
#define LCMA_BODY(T, GEMM)                                                          \
    if (m <= 0 || k <= 0 || n <= 0 || R <= 0) return 1;                             \
    if (M % m || K % k || N % n) return 1;                                          \
    const int64_t bm = M / m, bk = K / k, bn = N / n;                               \
    T *At = (T *)malloc(sizeof(T) * (size_t)(bm * bk));                             \
    T *Bt = (T *)malloc(sizeof(T) * (size_t)(bk * bn));                             \
    T *H = (T *)malloc(sizeof(T) * (size_t)R * (size_t)(bm * bn));                  \
    if (!At || !Bt || !H) { free(At); free(Bt); free(H); return 2; }                \
    for (int r = 0; r < R; ++r) {                                                   \
        memset(At, 0, sizeof(T) * (size_t)(bm * bk));                               \
        for (int i = 0; i < m; ++i)                                                 \
            for (int l = 0; l < k; ++l) {                                           \
                const int u = U[(r * m + i) * k + l];                               \
                if (!u) continue;                                                   \
                const T *Ab = A + (i * bm) * lda + l * bk;                          \
                for (int64_t x = 0; x < bm; ++x)                                    \
                    for (int64_t y = 0; y < bk; ++y)                                \
                        At[x * bk + y] += (T)u * Ab[x * lda + y];                   \
            }                                                                       \
        memset(Bt, 0, sizeof(T) * (size_t)(bk * bn));                               \
        for (int l = 0; l < k; ++l)                                                 \
            for (int j = 0; j < n; ++j) {                                           \
                const int v = V[(r * k + l) * n + j];                               \
                if (!v) continue;                                                   \
                const T *Bb = B + (l * bk) * ldb + j * bn;                          \
                for (int64_t y = 0; y < bk; ++y)                                    \
                    for (int64_t z = 0; z < bn; ++z)                                \
                        Bt[y * bn + z] += (T)v * Bb[y * ldb + z];                   \
            }                                                                       \
        GEMM(bm, bn, bk, At, bk, Bt, bn, H + (size_t)r * (size_t)(bm * bn), bn);    \
    }                                                                               \
    for (int i = 0; i < m; ++i)                                                     \
        for (int j = 0; j < n; ++j) {                                               \
            T *Cb = C + (i * bm) * ldc + j * bn;                                    \
            for (int64_t x = 0; x < bm; ++x)                                        \
                for (int64_t z = 0; z < bn; ++z) Cb[x * ldc + z] = (T)0;            \
            for (int r = 0; r < R; ++r) {                                           \
                const int w = W[(r * m + i) * n + j];                               \
                if (!w) continue;                                                   \
                const T *Hr = H + (size_t)r * (size_t)(bm * bn);                    \
                for (int64_t x = 0; x < bm; ++x)                                    \
                    for (int64_t z = 0; z < bn; ++z)                                \
                        Cb[x * ldc + z] += (T)w * Hr[x * bn + z];                   \
            }                                                                       \
        }                                                                           \
    free(At); free(Bt); free(H);                                                    \
    return 0;

int oracle_lcma_f64(int m, int k, int n, int R,
                    const int32_t *U, const int32_t *V, const int32_t *W,
                    int64_t M, int64_t N, int64_t K,
                    const double *A, int64_t lda,
                    const double *B, int64_t ldb,
                    double *C, int64_t ldc)
{
    LCMA_BODY(double, oracle_gemm_f64)
}

int oracle_lcma_i64(int m, int k, int n, int R,
                    const int32_t *U, const int32_t *V, const int32_t *W,
                    int64_t M, int64_t N, int64_t K,
                    const int64_t *A, int64_t lda,
                    const int64_t *B, int64_t ldb,
                    int64_t *C, int64_t ldc)
{
    LCMA_BODY(int64_t, oracle_gemm_i64)
}

/*
 * Brent identity.  Returns the number of violated equations and, when
 * first_bad is not NULL, stores the flat index of the first one in the
 * row-major order (i, a, b, j, c, d) with extents (m, k, k, n, m, n);
 * -1 when all hold.
 */
int64_t oracle_brent_residual(int m, int k, int n, int R,
                              const int32_t *U, const int32_t *V, const int32_t *W,
                              int64_t *first_bad)
{
    int64_t bad = 0, first = -1, idx = 0;
    for (int i = 0; i < m; ++i)
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b)
                for (int j = 0; j < n; ++j)
                    for (int c = 0; c < m; ++c)
                        for (int d = 0; d < n; ++d, ++idx) {
                            int64_t s = 0;
                            for (int r = 0; r < R; ++r)
                                s += (int64_t)U[(r * m + i) * k + a] *
                                     (int64_t)V[(r * k + b) * n + j] *
                                     (int64_t)W[(r * m + c) * n + d];
                            const int64_t want = (a == b && i == c && j == d) ? 1 : 0;
                            if (s != want) {
                                if (first < 0) first = idx;
                                ++bad;
                            }
                        }
    if (first_bad) *first_bad = first;
    return bad;
}
