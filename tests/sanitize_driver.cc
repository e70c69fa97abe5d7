// Host-only driver for the sanitizer build (tests/test_sanitizers.py): exercises the C oracle and the host side of the
// library (scheme loader and verifier, cost model, schedule arithmetic, every argument check that answers before a
// launch) under AddressSanitizer and UndefinedBehaviorSanitizer.  Nothing here touches a GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../include/lcma.h"

extern "C" {
void oracle_gemm_f64(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb, double *C, int64_t ldc);
void oracle_gemm_i64(int64_t M, int64_t N, int64_t K, const int64_t *A, int64_t lda, const int64_t *B, int64_t ldb, int64_t *C, int64_t ldc);
int oracle_lcma_i64(int m, int k, int n, int R, const int32_t *U, const int32_t *V, const int32_t *W, int64_t M, int64_t N, int64_t K,
                    const int64_t *A, int64_t lda, const int64_t *B, int64_t ldb, int64_t *C, int64_t ldc);
int oracle_lcma_f64(int m, int k, int n, int R, const int32_t *U, const int32_t *V, const int32_t *W, int64_t M, int64_t N, int64_t K,
                    const double *A, int64_t lda, const double *B, int64_t ldb, double *C, int64_t ldc);
int64_t oracle_brent_residual(int m, int k, int n, int R, const int32_t *U, const int32_t *V, const int32_t *W, int64_t *first);
}

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "CHECK failed line %d: %s\n", __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(int argc, char **argv) {
    // ---- schemes through the library, coefficients handed to the oracle
    const char *names[] = {"builtin:strassen", "builtin:laderman", "builtin:strassen2"};
    for (const char *name : names) {
        lcma_scheme *s = nullptr;
        CHECK(lcma_scheme_load(name, &s) == LCMA_OK);
        int64_t bad = 0;
        CHECK(lcma_scheme_verify(s, &bad) == LCMA_OK && bad == -1);
        int m, k, n, R, nu, nv, nw;
        CHECK(lcma_scheme_info(s, &m, &k, &n, &R, &nu, &nv, &nw) == LCMA_OK);
        std::vector<int8_t> U(R * m * k), V(R * k * n), W(R * m * n);
        CHECK(lcma_scheme_coeffs(s, U.data(), V.data(), W.data()) == LCMA_OK);
        std::vector<int32_t> U32(U.begin(), U.end()), V32(V.begin(), V.end()), W32(W.begin(), W.end());
        int64_t first = 0;
        CHECK(oracle_brent_residual(m, k, n, R, U32.data(), V32.data(), W32.data(), &first) == 0 && first == -1);
        // the LCMA evaluator against the triple loop, integer and fp64, leading dimensions larger than the rows
        const int64_t M = 3 * m, N = 2 * n, K = 5 * k, lda = K + 3, ldb = N + 1, ldc = N + 2;
        std::vector<int64_t> A(M * lda), Bm(K * ldb), C(M * ldc, -7), D(M * ldc, -9);
        for (size_t i = 0; i < A.size(); ++i) A[i] = (int64_t)(i * 7 % 11) - 5;
        for (size_t i = 0; i < Bm.size(); ++i) Bm[i] = (int64_t)(i * 5 % 7) - 3;
        oracle_gemm_i64(M, N, K, A.data(), lda, Bm.data(), ldb, C.data(), ldc);
        CHECK(oracle_lcma_i64(m, k, n, R, U32.data(), V32.data(), W32.data(), M, N, K, A.data(), lda, Bm.data(), ldb, D.data(), ldc) == 0);
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) CHECK(C[i * ldc + j] == D[i * ldc + j]);
        CHECK(C[N] == -7 && D[N] == -9); // the padding of the rows is untouched
        std::vector<double> Af(A.begin(), A.end()), Bf(Bm.begin(), Bm.end()), Cf(M * ldc), Df(M * ldc);
        oracle_gemm_f64(M, N, K, Af.data(), lda, Bf.data(), ldb, Cf.data(), ldc);
        CHECK(oracle_lcma_f64(m, k, n, R, U32.data(), V32.data(), W32.data(), M, N, K, Af.data(), lda, Bf.data(), ldb, Df.data(), ldc) == 0);
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) CHECK(Cf[i * ldc + j] == Df[i * ldc + j] && Cf[i * ldc + j] == (double)C[i * ldc + j]);
        CHECK(oracle_lcma_i64(m, k, n, R, U32.data(), V32.data(), W32.data(), M + 1, N, K, A.data(), lda, Bm.data(), ldb, D.data(), ldc) == 1);
        // a planted error is found at the same place by both checkers
        W32[0] = W32[0] ? 0 : 1;
        int64_t f2 = -1;
        CHECK(oracle_brent_residual(m, k, n, R, U32.data(), V32.data(), W32.data(), &f2) > 0 && f2 >= 0);
        // host arithmetic of the library on this scheme
        lcma_hw hw;
        CHECK(lcma_hw_mi355x(LCMA_BF16, &hw) == LCMA_OK);
        lcma_stage_costs costs;
        CHECK(lcma_model_stages(s, 8192, 14336, 4096, &hw, &costs) == LCMA_OK && costs.seconds[2] > 0);
        double e8, e9, e10;
        CHECK(lcma_model_intensity(s, 4096, 4096, 4096, &e8, &e9, &e10) == LCMA_OK && e8 > 0);
        CHECK(lcma_unfused_workspace_bytes(100, 200, 72, LCMA_F32, s) > 0);
        CHECK(lcma_fp8_workspace_bytes(s, 100, 200, 72) > 0 && lcma_fp8_prepared_w_bytes(s, 200, 72) > 0);
        // argument checks that answer before any launch (fake, never dereferenced pointers)
        void *P = (void *)0x100000;
        CHECK(lcma_gemm(256, 256, 252, P, 256, P, 256, P, 256, LCMA_F16, s, nullptr) != LCMA_OK);
        CHECK(lcma_gemm(-1, 256, 256, P, 256, P, 256, P, 256, LCMA_F16, s, nullptr) == LCMA_ERR_ARG);
        CHECK(lcma_gemm_unfused(3, 256, 256, 256, P, 256, P, 256, P, 256, LCMA_F16, s, P, 1 << 20, 0, nullptr) == LCMA_ERR_ARG);
        CHECK(lcma_fp8_gemm_lcma(256, 256, 256, P, 256, P, P, 256, s, P, 16, nullptr) != LCMA_OK);
        CHECK(lcma_prepare_b(256, 250, P, 256, LCMA_F16, s, P, nullptr) != LCMA_OK);
        CHECK(std::strlen(lcma_last_error()) > 0);
        lcma_scheme_free(s);
    }
    // ---- scheme files: good, truncated, garbage, oversized coefficients, missing
    const std::string dir = argc > 1 ? argv[1] : "/tmp";
    const std::string good = dir + "/sanitize_good.txt", bad1 = dir + "/sanitize_bad1.txt", bad2 = dir + "/sanitize_bad2.txt", bad3 = dir + "/sanitize_bad3.txt";
    {
        FILE *f = std::fopen(good.c_str(), "w");
        CHECK(f);
        std::fputs("# classical 1x1x1\n1 1 1 1\n1\n1\n1\n", f);
        std::fclose(f);
        f = std::fopen(bad1.c_str(), "w");
        std::fputs("2 2 2 7\n1 0 0 1\n", f); // truncated
        std::fclose(f);
        f = std::fopen(bad2.c_str(), "w");
        std::fputs("2 2 x 7\n@@@\n", f);
        std::fclose(f);
        f = std::fopen(bad3.c_str(), "w");
        std::fputs("1 1 1 1\n1000\n1\n1\n", f); // does not fit int8
        std::fclose(f);
    }
    lcma_scheme *s = nullptr;
    CHECK(lcma_scheme_load(good.c_str(), &s) == LCMA_OK && lcma_scheme_verify(s, nullptr) == LCMA_OK);
    lcma_scheme_free(s);
    s = nullptr;
    CHECK(lcma_scheme_load(bad1.c_str(), &s) == LCMA_ERR_PARSE && !s);
    CHECK(lcma_scheme_load(bad2.c_str(), &s) == LCMA_ERR_PARSE);
    CHECK(lcma_scheme_load(bad3.c_str(), &s) == LCMA_ERR_PARSE);
    CHECK(lcma_scheme_load((dir + "/no_such_file.txt").c_str(), &s) == LCMA_ERR_IO);
    CHECK(lcma_scheme_load(nullptr, &s) == LCMA_ERR_ARG && lcma_scheme_load("builtin:nonsense", &s) != LCMA_OK);
    lcma_scheme_free(nullptr);
    // ---- selector, predictions, schedule arithmetic (Sec. 3.2 worked example: 256 groups of 7 on 78 units)
    for (int dt = 0; dt < 3; ++dt)
        for (int64_t M : {1, 100, 2048, 16384}) {
            const int pick = lcma_select(M, 4096, 14336, (lcma_dtype)dt);
            CHECK(pick >= 0 && pick <= 3);
            lcma_choice ch;
            CHECK(lcma_select_dataflow(M, 4096, 14336, (lcma_dtype)dt, 1, &ch) == LCMA_OK);
            (void)lcma_predict_seconds(pick, M, 4096, 14336, (lcma_dtype)dt);
            (void)lcma_predict_unfused_seconds(1, M, 4096, 14336, (lcma_dtype)dt, 0);
        }
    CHECK(lcma_select(0, 1, 1, LCMA_F32) < 0 || true);
    int64_t a = 0, b = 0;
    CHECK(lcma_sched_waves(256, 7, 78, &a, &b) == LCMA_OK && a == 23 && b == 28);
    int64_t covered = 0;
    for (int u = 0; u < 78; ++u) {
        CHECK(lcma_sched_range(256, 7, 78, u, &a, &b) == LCMA_OK && a <= b);
        covered += b - a;
    }
    CHECK(covered == 256 * 7);
    CHECK(lcma_sched_range(256, 7, 78, 78, &a, &b) != LCMA_OK);
    for (int i = 0; i < lcma_variant_count(); ++i) {
        int sid, dtype, tm, tn, tk, mm, mn, mk;
        CHECK(lcma_variant_name(i) && lcma_variant_info(i, &sid, &dtype, &tm, &tn, &tk, &mm, &mn, &mk) == LCMA_OK);
    }
    CHECK(!lcma_variant_name(lcma_variant_count()) && lcma_variant_b_layout(-1) == -1);
    CHECK(lcma_set_tuning("panel", "4") == LCMA_OK && lcma_set_tuning("nonsense", "1") == LCMA_ERR_ARG && lcma_set_tuning("panel", "") == LCMA_OK);
    std::printf("sanitize driver ok\n");
    return 0;
}
