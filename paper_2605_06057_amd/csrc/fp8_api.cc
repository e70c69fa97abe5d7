// Host side of the FP8 path (paper Sec. 4.1: bf16 operands quantised to FP8 E4M3 with 1 x 128 block scaling; Sec. 4.3:
// the quantisation fused into the Combine A stage): argument checks, geometry of the planes, launches.
#include "host_common.h"

#include <cstring>

extern "C" int lcma_launch_fp8_quantize_rows(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream);

namespace lcma {
namespace {

int64_t round_up(int64_t x, int64_t g) { return (x + g - 1) / g * g; }
const int64_t kLim = (int64_t)1 << 31;

// Planes of the LCMA form: blocks padded to 128 rows and to whole scale blocks along K.
struct Fp8Geometry {
    int64_t bm, bn, bk, ls;           // rows of At_r, rows of Bt_r^T, columns (bytes) of both, scale pitch
    int64_t aq, as, h, wq, ws;        // byte sizes (each a multiple of 256)
};
Fp8Geometry fp8_geometry(const lcma_scheme &s, int64_t M, int64_t N, int64_t K) {
    Fp8Geometry g;
    g.bm = round_up((M + s.m - 1) / s.m, 128);
    g.bn = round_up((N + s.n - 1) / s.n, 128);
    g.bk = round_up((K + s.k - 1) / s.k, 128);
    g.ls = round_up(g.bk / 128, 4);
    g.aq = round_up((int64_t)s.R * g.bm * g.bk, 256);
    g.as = round_up((int64_t)s.R * g.bm * g.ls, 256);
    g.h = round_up((int64_t)s.R * g.bm * g.bn * 2, 256);
    g.wq = round_up((int64_t)s.R * g.bn * g.bk, 256);
    g.ws = round_up((int64_t)s.R * g.bn * g.ls, 256);
    return g;
}

const Fp8Kernel *find_fp8(int scheme_id) {
    for (int i = 0; i < kFp8KernelCount; ++i)
        if (kFp8Kernels[i].launch_comb_a && kFp8Kernels[i].scheme_id == scheme_id) return &kFp8Kernels[i];
    return nullptr;
}

const StageKernel *find_stage_bf16(int scheme_id) {
    for (int i = 0; i < kStageKernelCount; ++i)
        if (kStageKernels[i].launch_comb_h && kStageKernels[i].scheme_id == scheme_id && kStageKernels[i].dtype == LCMA_BF16)
            return &kStageKernels[i];
    return nullptr;
}

lcma_status fp8_scheme(const lcma_scheme *scheme, const char *who, const Fp8Kernel **fk) {
    if (!scheme) return fail(LCMA_ERR_ARG, "%s: a scheme is required", who);
    if (const lcma_status st = lcma_scheme_verify(scheme, nullptr)) return st;
    *fk = scheme->builtin ? find_fp8(scheme->builtin) : nullptr;
    if (!*fk || !find_stage_bf16(scheme->builtin))
        return fail(LCMA_ERR_NOKERNEL, "%s: no FP8 kernels were generated for scheme <%d,%d,%d;%d>", who, scheme->m,
                    scheme->k, scheme->n, scheme->R);
    return LCMA_OK;
}

} // namespace
} // namespace lcma

using namespace lcma;

extern "C" int64_t lcma_fp8_code_pitch(int64_t K) { return K > 0 ? round_up(K, 128) : -1; }
extern "C" int64_t lcma_fp8_scale_pitch(int64_t K) { return K > 0 ? round_up(round_up(K, 128) / 128, 4) : -1; }

extern "C" lcma_status lcma_fp8_quantize(int64_t rows, int64_t K, const void *X, int64_t ldx, void *Q, void *S, void *stream) {
    const char *who = "lcma_fp8_quantize";
    if (rows < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (rows == 0 || K == 0) return LCMA_OK;
    if (!X || !Q || !S) return fail(LCMA_ERR_ARG, "%s: null pointer", who);
    if (ldx < K) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)X | (uintptr_t)Q) & 15) || ((uintptr_t)S & 3) || ((ldx * 2) & 15))
        return fail(LCMA_ERR_ARG, "%s: X and Q must be 16-byte aligned, S 4-byte aligned, ldx a multiple of 8", who);
    if (K % 8) return fail(LCMA_ERR_SHAPE, "%s: K = %lld must be a multiple of 8 (16 bytes of bf16)", who, (long long)K);
    const int64_t kp = round_up(K, 128), ls = round_up(kp / 128, 4);
    if (((rows - 1) * ldx + kp) * 2 >= kLim || rows * kp >= kLim) return fail(LCMA_ERR_SHAPE, "%s: a matrix spans 2 GiB or more", who);
    if ((rows + 15) / 16 > 65535) return fail(LCMA_ERR_SHAPE, "%s: too many rows", who); // (the y dimension of the grid)
    Fp8QuantParams p;
    std::memset(&p, 0, sizeof p);
    p.X = X;
    p.Q = Q;
    p.S = S;
    p.x_bytes = (uint32_t)(((rows - 1) * ldx + K) * 2);
    p.q_bytes = (uint32_t)(rows * kp);
    p.s_bytes = (uint32_t)(rows * ls);
    p.ldx_b = (uint32_t)(ldx * 2);
    p.ldq_b = (uint32_t)kp;
    p.lds_b = (uint32_t)ls;
    p.k_row_b = (uint32_t)(K * 2);
    p.rows = (int32_t)rows;
    if (const int err = lcma_launch_fp8_quantize_rows(&p, (int)((rows + 15) / 16), (int)(kp / 128), stream))
        return fail(LCMA_ERR_HIP, "%s: launch failed with HIP error %d", who, err);
    return LCMA_OK;
}

extern "C" lcma_status lcma_fp8_gemm_nt(int64_t M, int64_t N, int64_t K, const void *Aq, const void *Sa, const void *Wq,
                                        const void *Sw, void *C, int64_t ldc, void *stream) {
    const char *who = "lcma_fp8_gemm_nt";
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (M == 0 || N == 0) return LCMA_OK;
    if (K == 0) return empty_product(M, N, C, ldc, LCMA_BF16, 0.f, stream);
    if (!Aq || !Sa || !Wq || !Sw || !C) return fail(LCMA_ERR_ARG, "%s: null pointer", who);
    if (ldc < N) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)Aq | (uintptr_t)Wq | (uintptr_t)C) & 15) || (((uintptr_t)Sa | (uintptr_t)Sw) & 3) || ((ldc * 2) & 15))
        return fail(LCMA_ERR_ARG, "%s: code matrices and C must be 16-byte aligned (ldc a multiple of 8), scale matrices 4-byte aligned", who);
    if (K % 8 || N % 8) return fail(LCMA_ERR_SHAPE, "%s: N = %lld and K = %lld must be multiples of 8", who, (long long)N, (long long)K);
    const int64_t kp = round_up(K, 128), ls = round_up(kp / 128, 4);
    if ((round_up(M, 256) * kp) >= kLim || (round_up(N, 256) * kp) >= kLim || ((round_up(M, 256) - 1) * ldc + round_up(N, 256)) * 2 >= kLim)
        return fail(LCMA_ERR_SHAPE, "%s: a matrix spans 2 GiB or more", who);
    PlaneGemmParams p;
    std::memset(&p, 0, sizeof p);
    p.A = Aq;
    p.SA = Sa;
    p.B = Wq;
    p.SB = Sw;
    p.C = C;
    p.a_bytes = (uint32_t)(M * kp);
    p.sa_bytes = (uint32_t)(M * ls);
    p.b_bytes = (uint32_t)(N * kp);
    p.sb_bytes = (uint32_t)(N * ls);
    p.c_bytes = (uint32_t)(((M - 1) * ldc + N) * 2);
    p.lda_b = p.ldb_b = (uint32_t)kp;
    p.lsa_b = p.lsb_b = (uint32_t)ls;
    p.ldc_b = (uint32_t)(ldc * 2);
    p.ny = (int32_t)(kp / 128);
    p.n_row_b = (uint32_t)(N * 2);
    return plane_gemm(who, PG_FP8_BF16, p, 1, M, N, 0, 1, nullptr, 0, stream);
}

extern "C" int64_t lcma_fp8_prepared_w_bytes(const lcma_scheme *scheme, int64_t N, int64_t K) {
    if (!scheme || N <= 0 || K <= 0) return -1;
    const Fp8Geometry g = fp8_geometry(*scheme, 1, N, K);
    return g.wq + g.ws;
}

extern "C" int64_t lcma_fp8_workspace_bytes(const lcma_scheme *scheme, int64_t M, int64_t N, int64_t K) {
    if (!scheme || M <= 0 || N <= 0 || K <= 0) return -1;
    const Fp8Geometry g = fp8_geometry(*scheme, M, N, K);
    return g.aq + g.as + g.h + plane_gemm_scratch_bytes(256);
}

namespace {
// Combine (A or W) with the quantisation fused in: rows x K bf16 matrix X cut into `grid_rows` x `grid_k` blocks of
// (padded) brows x bk, planes written to Q / S.
lcma_status combine_quantize(const char *who, int (*launch)(const Fp8QuantParams *, int, int, void *), int R, int64_t rows,
                             int64_t K, const void *X, int64_t ldx, int64_t brows, int64_t bk, int64_t ls, int grid_rows,
                             int grid_k, void *Q, void *S, void *stream) {
    if (((grid_rows * brows - 1) * ldx + grid_k * bk) * 2 >= kLim || (int64_t)R * brows * bk >= kLim)
        return fail(LCMA_ERR_SHAPE, "%s: a matrix or a set of planes spans 2 GiB or more", who);
    if (brows / 16 > 65535) return fail(LCMA_ERR_SHAPE, "%s: too many rows", who); // (the y dimension of the grid)
    Fp8QuantParams p;
    std::memset(&p, 0, sizeof p);
    p.X = X;
    p.Q = Q;
    p.S = S;
    p.x_bytes = (uint32_t)(((rows - 1) * ldx + K) * 2);
    p.q_bytes = (uint32_t)((int64_t)R * brows * bk);
    p.s_bytes = (uint32_t)((int64_t)R * brows * ls);
    p.ldx_b = (uint32_t)(ldx * 2);
    p.x_brow = (uint32_t)(brows * ldx * 2);
    p.x_bcol = (uint32_t)(bk * 2);
    p.ldq_b = (uint32_t)bk;
    p.lds_b = (uint32_t)ls;
    p.q_plane = (uint32_t)(brows * bk);
    p.s_plane = (uint32_t)(brows * ls);
    p.k_row_b = (uint32_t)(K * 2);
    p.rows = (int32_t)brows;
    if (const int err = launch(&p, (int)(brows / 16), (int)(bk / 128), stream))
        return fail(LCMA_ERR_HIP, "%s: launch failed with HIP error %d", who, err);
    return LCMA_OK;
}
} // namespace

extern "C" lcma_status lcma_fp8_prepare_w(int64_t N, int64_t K, const void *W, int64_t ldw, const lcma_scheme *scheme,
                                          void *Wp, void *stream) {
    const char *who = "lcma_fp8_prepare_w";
    const Fp8Kernel *fk = nullptr;
    if (const lcma_status st = fp8_scheme(scheme, who, &fk)) return st;
    if (N < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (N == 0 || K == 0) return LCMA_OK;
    if (!W || !Wp) return fail(LCMA_ERR_ARG, "%s: null pointer", who);
    if (ldw < K) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)W) & 15) || ((uintptr_t)Wp & 255) || ((ldw * 2) & 15))
        return fail(LCMA_ERR_ARG, "%s: W must be 16-byte aligned with ldw a multiple of 8, Wp 256-byte aligned", who);
    if (K % 8) return fail(LCMA_ERR_SHAPE, "%s: K = %lld must be a multiple of 8", who, (long long)K);
    const Fp8Geometry g = fp8_geometry(*scheme, 1, N, K);
    return combine_quantize(who, fk->launch_prep_w, scheme->R, N, K, W, ldw, g.bn, g.bk, g.ls, scheme->n, scheme->k, Wp,
                            (char *)Wp + g.wq, stream);
}

extern "C" lcma_status lcma_fp8_gemm_lcma(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *Wp,
                                          void *C, int64_t ldc, const lcma_scheme *scheme, void *workspace,
                                          int64_t workspace_bytes, void *stream) {
    const char *who = "lcma_fp8_gemm_lcma";
    const Fp8Kernel *fk = nullptr;
    if (const lcma_status st = fp8_scheme(scheme, who, &fk)) return st;
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (M == 0 || N == 0) return LCMA_OK;
    if (K == 0) return empty_product(M, N, C, ldc, LCMA_BF16, 0.f, stream);
    if (!A || !Wp || !C || !workspace) return fail(LCMA_ERR_ARG, "%s: null pointer", who);
    if (lda < K || ldc < N) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)A | (uintptr_t)C) & 15) || (((uintptr_t)Wp | (uintptr_t)workspace) & 255) || ((lda * 2) & 15) || ((ldc * 2) & 15))
        return fail(LCMA_ERR_ARG, "%s: A and C must be 16-byte aligned with leading dimensions multiples of 8, Wp and the "
                                  "workspace 256-byte aligned", who);
    if (K % 8 || N % 8) return fail(LCMA_ERR_SHAPE, "%s: N = %lld and K = %lld must be multiples of 8", who, (long long)N, (long long)K);
    const Fp8Geometry g = fp8_geometry(*scheme, M, N, K);
    const int64_t need = g.aq + g.as + g.h + plane_gemm_scratch_bytes(256);
    if (workspace_bytes < need)
        return fail(LCMA_ERR_ARG, "%s: the workspace holds %lld bytes, %lld are needed", who, (long long)workspace_bytes,
                    (long long)need);
    const int R = scheme->R;
    if (g.aq >= kLim || g.wq >= kLim || g.h >= kLim || ((g.bm * scheme->m - 1) * ldc + g.bn * scheme->n) * 2 >= kLim)
        return fail(LCMA_ERR_SHAPE, "%s: a matrix or a set of planes spans 2 GiB or more", who);
    if (g.bm / 16 > 65535) return fail(LCMA_ERR_SHAPE, "%s: M is too large", who); // (rows: the y dimension of Combine H's grid)
    char *Aq = (char *)workspace, *Sa = Aq + g.aq, *H = Sa + g.as;
    const char *Wq = (const char *)Wp, *Sw = Wq + g.wq;
    // stage 1: Combine A (Eq. 3) with the quantisation fused in
    if (const lcma_status st = combine_quantize(who, fk->launch_comb_a, R, M, K, A, lda, g.bm, g.bk, g.ls, scheme->m,
                                                scheme->k, Aq, Sa, stream))
        return st;
    // stage 3: the R products H_r = At_r x Bt_r (Eq. 5) as one batched launch on the codes, product-major order
    PlaneGemmParams p;
    std::memset(&p, 0, sizeof p);
    p.A = Aq;
    p.SA = Sa;
    p.B = Wq;
    p.SB = Sw;
    p.C = H;
    p.a_bytes = (uint32_t)((int64_t)R * g.bm * g.bk);
    p.sa_bytes = (uint32_t)((int64_t)R * g.bm * g.ls);
    p.b_bytes = (uint32_t)((int64_t)R * g.bn * g.bk);
    p.sb_bytes = (uint32_t)((int64_t)R * g.bn * g.ls);
    p.c_bytes = (uint32_t)((int64_t)R * g.bm * g.bn * 2);
    p.lda_b = p.ldb_b = (uint32_t)g.bk;
    p.lsa_b = p.lsb_b = (uint32_t)g.ls;
    p.ldc_b = (uint32_t)(g.bn * 2);
    p.a_plane = (uint32_t)(g.bm * g.bk);
    p.sa_plane = (uint32_t)(g.bm * g.ls);
    p.b_plane = (uint32_t)(g.bn * g.bk);
    p.sb_plane = (uint32_t)(g.bn * g.ls);
    p.c_plane = (uint32_t)(g.bm * g.bn * 2);
    p.ny = (int32_t)(g.bk / 128);
    p.n_row_b = (uint32_t)(g.bn * 2);
    if (const lcma_status st = plane_gemm(who, PG_FP8_F16, p, R, g.bm, g.bn, 0, 0, H + g.h, plane_gemm_scratch_bytes(256), stream))
        return st;
    // stage 4: Combine H (Eq. 6): fp32 sums of the fp16 products in ascending r, one rounding to bf16
    const StageKernel *sk = find_stage_bf16(scheme->builtin);
    CombHParams h;
    h.H = H;
    h.C = C;
    h.h_bytes = p.c_bytes;
    h.c_bytes = (uint32_t)(((M - 1) * ldc + N) * 2);
    h.h_ld_b = (uint32_t)(g.bn * 2);
    h.h_plane_b = (uint32_t)(g.bm * g.bn * 2);
    h.ldc_b = (uint32_t)(ldc * 2);
    h.c_brow = (uint32_t)(g.bm * ldc * 2);
    h.c_bcol = (uint32_t)(g.bn * 2);
    h.n_row_b = (uint32_t)(N * 2);
    const int64_t gy = (g.bn * 2 + 255) / 256;
    if (const int err = sk->launch_comb_h(&h, (int)(g.bm / 16), (int)gy, stream))
        return fail(LCMA_ERR_HIP, "%s: Combine-H launch failed with HIP error %d", who, err);
    return LCMA_OK;
}
