// The dataflows the paper starts from, on gfx950, so that they can be measured against the fused
// kernels (the step-wise ablation of Sec. 4.5):
//   level 1  Algorithm 1: Combine A, Combine B, R block products and Combine H as four stages, each
//            reading its operands from and writing its result to device memory;
//   level 2  Algorithm 2 as printed: Combine A and Combine B write At_r, Bt_r to device memory, one
//            kernel multiplies them group by group and applies W on chip (H_r never leaves the chip).
// (lcma_gemm is the third step: nothing but C is written.)  Everything lives in a caller-provided
// workspace: the planes At (R x bm x bk), Bt (R x bn x bk) and, for level 1, H (R x bm x bn), in
// the type the products are multiplied in, with bm, bn multiples of 128 and bk of 64 elements (16 for
// fp32) that cover ceil(M/m), ceil(N/n), ceil(K/k); the padding holds zeros.
#include "host_common.h"

#include <cmath>
#include <cstdlib>
#include <cstring>

namespace lcma {
namespace {

int64_t round_up(int64_t x, int64_t g) { return (x + g - 1) / g * g; }
int64_t align256(int64_t x) { return round_up(x, 256); }

struct Geometry {
    int64_t bm, bn, bk, es, h_es; // h_es: element size of the planes of products (level 1)
    int64_t at_bytes, bt_bytes, h_bytes; // each rounded up to 256
    int64_t total() const { return at_bytes + bt_bytes + h_bytes; }
};

// planes: what the stage kernels of (scheme, dtype) work on (StageKernel::planes), R without stage kernels
int planes_of(const lcma_scheme &s, int dtype);
Geometry geometry(const lcma_scheme &s, int64_t M, int64_t N, int64_t K, int dtype) {
    Geometry g;
    const int64_t R = planes_of(s, dtype);
    g.es = dtype_size(dtype);
    const int64_t kg = g.es == 4 ? 16 : 64;
    g.bm = round_up((M + s.m - 1) / s.m, 128);
    g.bn = round_up((N + s.n - 1) / s.n, 128);
    g.bk = round_up((K + s.k - 1) / s.k, kg);
    g.at_bytes = align256(R * g.bm * g.bk * g.es);
    g.bt_bytes = align256(R * g.bn * g.bk * g.es);
    // fp16 storage: the products are kept in fp32 (fp16 planes would carry no more bits than C itself and put the
    // result past four times the plain kernel's error); bf16 storage keeps them in fp16, fp32 storage in fp32
    g.h_es = dtype == LCMA_F16 ? 4 : g.es;
    g.h_bytes = align256(R * g.bm * g.bn * g.h_es);
    return g;
}

const StageKernel *find_stage(int scheme_id, int dtype) {
    for (int i = 0; i < kStageKernelCount; ++i)
        if (kStageKernels[i].launch_comb_a && kStageKernels[i].scheme_id == scheme_id && kStageKernels[i].dtype == dtype)
            return &kStageKernels[i];
    return nullptr;
}
int planes_of(const lcma_scheme &s, int dtype) {
    const StageKernel *sk = s.builtin ? find_stage(s.builtin, dtype) : nullptr;
    return sk ? sk->planes : s.R;
}

// Seconds of the GEMM stage with kernel v on planes of geometry g: R tile-jobs per tile position for the
// batched plain kernel, one group of R products for the Algorithm 2 kernel, in rounds of 256 * occupancy
// work-groups.  A round costs its MFMA flops at the kernel's measured fraction of the peak (`eff` of a
// batched kernel is the slope of its round time over K) plus a fixed part for filling the pipeline and
// writing the tiles out: 6.4 us for 128 KB of output per CU (measured on the 256 x 256 fp16 kernel,
// K/k = 2048 against K = 4096), taken proportional to the bytes a CU writes per round.
double gemm_stage_seconds(const Variant &v, int R, const Geometry &g) {
    const double peak = v.dtype == LCMA_F32 ? 157.3e12 : 2516.6e12, slots = 256.0 * v.occ;
    const double tiles = (double)(g.bm / v.TM) * (double)(g.bn / v.TN);
    const double jobs = v.batch ? tiles * R : tiles, flops_per_job = 2.0 * v.TM * v.TN * (double)g.bk * (v.batch ? 1 : R);
    const double t_round = slots * flops_per_job / (v.eff * peak) +
                           (v.batch ? 6.4e-6 * (double)(v.TM * v.TN * dtype_size(v.dtype) * v.occ) / 131072.0 : 0.0);
    const double full = std::floor(jobs / slots), rest = jobs - full * slots;
    return (full + (rest > 0 ? ((v.occ > 1 && rest <= 256) ? 0.63 : 1.0) : 0.0)) * t_round;
}

// The stage kernel of the wanted kind with the smallest predicted time among those that divide the planes.
const Variant *find_gemm(bool batch, int scheme_id, int dtype, int R, const Geometry &g) {
    const Variant *best = nullptr;
    double best_t = 0.0;
    const Variant *force = forced_unfused_variant(); // ablation override
    for (int i = 0; i < kVariantCount; ++i) {
        const Variant &v = kVariants[i];
        if ((batch ? !v.batch : !v.left_planes) || v.scheme_id != scheme_id || v.dtype != dtype) continue;
        if (g.bm % v.TM || g.bn % v.TN || g.bk % v.TK) continue;
        if (force == &v) return &v;
        const double t = gemm_stage_seconds(v, R, g);
        if (!best || t < best_t) {
            best = &v;
            best_t = t;
        }
    }
    return best;
}

const double kLaunch = 2.0e-6; // seconds per launch of a stage (the launches of one call follow each other on one stream)

} // namespace
} // namespace lcma

using namespace lcma;

extern "C" int64_t lcma_unfused_workspace_bytes(int64_t M, int64_t N, int64_t K, lcma_dtype dtype, const lcma_scheme *scheme) {
    if (!scheme || !dtype_size(dtype) || M <= 0 || N <= 0 || K <= 0) return -1;
    return geometry(*scheme, M, N, K, dtype).total();
}

extern "C" int64_t lcma_split_group_scratch_bytes(void) { return plane_gemm_scratch_bytes(256); }

// Algorithm 1 priced stage by stage: the three memory-bound kernels at the rates measured for the scheme, the
// batched GEMM in rounds of work-groups.
extern "C" double lcma_predict_unfused_seconds(int scheme_id, int64_t M, int64_t N, int64_t K, lcma_dtype dtype,
                                               int combine_b_offline) {
    const int es = dtype_size(dtype);
    const lcma_scheme *s = builtin_scheme(scheme_id);
    const StageKernel *sk = find_stage(scheme_id, dtype);
    if (!es || !s || M <= 0 || N <= 0 || K <= 0 || !sk) return -1.0;
    const Geometry g = geometry(*s, M, N, K, dtype);
    const Variant *gemm = find_gemm(true, LCMA_PLAIN, dtype == LCMA_F32 ? LCMA_F32 : LCMA_F16, sk->planes, g);
    if (!gemm) return -1.0;
    const double R = sk->planes, dM = (double)M, dN = (double)N, dK = (double)K;
    const double at = R * g.bm * g.bk, bt = R * g.bn * g.bk, h = R * g.bm * g.bn; // elements of the planes
    double t = (dM * dK + at) * es / sk->rate_a + kLaunch;
    if (!combine_b_offline) t += (dK * dN + bt) * es / sk->rate_b + kLaunch;
    // 16-bit: the plane GEMM runs the stage (priced without the scratch of the Split-Group schedule, which only a
    // workspace larger than lcma_unfused_workspace_bytes() provides)
    const double t_planes = es == 2 ? plane_gemm_seconds(sk->planes, g.bm, g.bn, (int)(g.bk * es / 128), 0) : -1.0;
    t += (t_planes > 0.0 ? t_planes : gemm_stage_seconds(*gemm, sk->planes, g)) + kLaunch;
    t += (h * g.h_es + dM * dN * es) / sk->rate_h + kLaunch;
    return t;
}

extern "C" lcma_status lcma_select_dataflow(int64_t M, int64_t N, int64_t K, lcma_dtype dtype, int combine_b_offline,
                                            lcma_choice *out) {
    if (!out) return fail(LCMA_ERR_ARG, "lcma_select_dataflow: null output");
    if (!dtype_size(dtype)) return fail(LCMA_ERR_DTYPE, "lcma_select_dataflow: unknown dtype %d", (int)dtype);
    if (M <= 0 || N <= 0 || K <= 0) return fail(LCMA_ERR_ARG, "lcma_select_dataflow: bad shape");
    out->scheme_id = LCMA_PLAIN;
    out->dataflow = 0;
    out->seconds = lcma_predict_seconds(LCMA_PLAIN, M, N, K, dtype);
    for (int id = LCMA_STRASSEN; id <= LCMA_LADERMAN; ++id) {
        const double fused = lcma_predict_seconds(id, M, N, K, dtype);
        const double unfused = lcma_predict_unfused_seconds(id, M, N, K, dtype, combine_b_offline);
        if (fused > 0.0 && (out->seconds <= 0.0 || fused < out->seconds)) *out = lcma_choice{id, 0, fused};
        if (unfused > 0.0 && (out->seconds <= 0.0 || unfused < out->seconds)) *out = lcma_choice{id, 1, unfused};
    }
    return LCMA_OK;
}

extern "C" lcma_status lcma_gemm_unfused(int level, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                                         const void *B, int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype,
                                         const lcma_scheme *scheme, void *workspace, int64_t workspace_bytes,
                                         int reuse_bt, void *stream) {
    return gemm_unfused("lcma_gemm_unfused", level, M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, workspace,
                        workspace_bytes, reuse_bt, stream);
}

// fp16 storage: the combinations At_r and Bt_r that Algorithm 1 stores in fp16 have as many bits as the inputs, so a sum of
// many blocks loses relatively more than C's own rounding; with rows of up to 7 blocks (<3,3,3;23>) the result lands at
// 4.04 times the plain kernel's error on uniform and normal inputs (measured, and the CPU model of the dataflow gives the
// same figure), past the bound of 4 this library promises; with rows of up to 4 blocks it stays below 3.
static bool stored_combinations_meet_the_bound(const lcma_scheme &s, lcma_dtype dtype) {
    if (dtype != LCMA_F16) return true;
    // (stage kernels that multiply the rounding residuals of the worst combinations as well are inside the bound)
    if (const StageKernel *sk = s.builtin ? find_stage(s.builtin, dtype) : nullptr)
        if (sk->planes > s.R) return true;
    auto longest_row = [&](const std::vector<int8_t> &T, int per_row) {
        int most = 0;
        for (int r = 0; r < s.R; ++r) {
            int nnz = 0;
            for (int e = 0; e < per_row; ++e) nnz += T[(size_t)r * per_row + e] != 0;
            most = nnz > most ? nnz : most;
        }
        return most;
    };
    return longest_row(s.U, s.m * s.k) <= 4 && longest_row(s.V, s.k * s.n) <= 4;
}

// lcma_gemm / lcma_gemm_nt with a workspace: the fused kernel or Algorithm 1, whichever the time model predicts faster for
// the shape; without a scheme the plain product, for N x K weights on the plane GEMM.
extern "C" lcma_status lcma_gemm_ws(int b_layout, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                                    int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                                    void *workspace, int64_t workspace_bytes, int *dataflow, void *stream) {
    if (dataflow) *dataflow = 0;
    if (b_layout != 0 && b_layout != 2) return fail(LCMA_ERR_ARG, "lcma_gemm_ws: b_layout must be 0 (B is K x N) or 2 (W is N x K)");
    const bool nk = b_layout == 2;
    auto fused = [&]() {
        if (!nk) return lcma_gemm(M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, stream);
        if (!scheme) return lcma_gemm_nt_ws(M, N, K, A, lda, B, ldb, C, ldc, dtype, workspace, workspace ? workspace_bytes : 0, stream);
        return lcma_gemm_nt(M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, stream);
    };
    const int id = scheme ? scheme->builtin : 0;
    bool alg1 = false;
    if (id && workspace && !((uintptr_t)workspace & 255) && dtype_size(dtype) && M > 0 && N > 0 && K > 0 &&
        find_stage(id, dtype) && stored_combinations_meet_the_bound(*scheme, dtype) &&
        workspace_bytes >= geometry(*scheme, M, N, K, dtype).total()) {
        const double t_fused = lcma_predict_seconds(id, M, N, K, dtype), t_alg1 = lcma_predict_unfused_seconds(id, M, N, K, dtype, 0);
        alg1 = t_alg1 > 0.0 && (t_fused <= 0.0 || t_alg1 < t_fused);
    }
    if (!alg1) return fused();
    const lcma_status st = gemm_unfused("lcma_gemm_ws", 1, M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, workspace, workspace_bytes, 0,
                                        stream, nk);
    // shapes that only the fused kernels take (no whole 16-byte vectors along K, ...) fall back to them
    if (st == LCMA_ERR_SHAPE) return fused();
    if (st == LCMA_OK && dataflow) *dataflow = 1;
    return st;
}

lcma_status lcma::gemm_unfused(const char *who, int level, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                               const void *B, int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                               void *workspace, int64_t workspace_bytes, int reuse_bt, void *stream, bool b_nk) {
    const int es = dtype_size(dtype);
    if (!es) return fail(LCMA_ERR_DTYPE, "%s: unknown dtype %d", who, (int)dtype);
    if (level != 1 && level != 2) return fail(LCMA_ERR_ARG, "%s: level must be 1 (Algorithm 1) or 2 (Algorithm 2)", who);
    if (!scheme) return fail(LCMA_ERR_ARG, "%s: a scheme is required", who);
    if (const lcma_status st = lcma_scheme_verify(scheme, nullptr)) return st;
    const int id = scheme->builtin;
    const StageKernel *sk = id ? find_stage(id, dtype) : nullptr;
    if (!sk)
        return fail(LCMA_ERR_NOKERNEL, "%s: no stage kernels were generated for scheme <%d,%d,%d;%d> with dtype %d", who,
                    scheme->m, scheme->k, scheme->n, scheme->R, (int)dtype);
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (M == 0 || N == 0) return LCMA_OK;
    if (K == 0) return empty_product(M, N, C, ldc, dtype, 0.f, stream);
    if (!A || !B || !C || !workspace) return fail(LCMA_ERR_ARG, "%s: null pointer", who);
    // (b_nk: B is the N x K weight matrix W, rows k-contiguous, and the product is A W^T)
    if (lda < K || ldb < (b_nk ? K : N) || ldc < N) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15) || ((uintptr_t)workspace & 255))
        return fail(LCMA_ERR_ARG, "%s: matrix pointers must be 16-byte aligned, the workspace 256-byte aligned", who);
    if (((lda * es) | (ldb * es) | (ldc * es)) & 15)
        return fail(LCMA_ERR_ARG, "%s: leading dimensions must be multiples of 16 bytes", who);
    const int vec = 16 / es;
    if (N % vec || K % vec)
        return fail(LCMA_ERR_SHAPE, "%s: N = %lld and K = %lld must be multiples of %d (16 bytes of elements)", who,
                    (long long)N, (long long)K, vec);
    const Geometry g = geometry(*scheme, M, N, K, dtype);
    if (workspace_bytes < g.total())
        return fail(LCMA_ERR_ARG, "%s: the workspace holds %lld bytes, %lld are needed", who, (long long)workspace_bytes,
                    (long long)g.total());
    // level 1 works on the planes of the stage kernels (R, or more with compensated products); level 2 on the first R
    const int R = level == 1 ? sk->planes : scheme->R;
    const int64_t lim = (int64_t)1 << 31;
    const int64_t Mp = g.bm * scheme->m, Np = g.bn * scheme->n, Kp = g.bk * scheme->k;
    if (g.at_bytes >= lim || g.bt_bytes >= lim || g.h_bytes >= lim || ((Mp - 1) * lda + Kp) * es >= lim ||
        (b_nk ? (Np - 1) * ldb + Kp : (Kp - 1) * ldb + Np) * es >= lim || ((Mp - 1) * ldc + Np) * es >= lim)
        return fail(LCMA_ERR_SHAPE, "%s: a matrix or a set of planes spans 2 GiB or more", who);
    // Bt first: its place and size depend on N and K alone, so the planes of static weights stay where they are
    // when the number of rows M changes between calls
    char *Bt = (char *)workspace, *At = Bt + g.bt_bytes, *H = At + g.at_bytes;
    // the products are multiplied in fp16 for both 16-bit storage types
    const int ct = dtype == LCMA_F32 ? LCMA_F32 : LCMA_F16;
    const Variant *gemm = level == 1 ? find_gemm(true, LCMA_PLAIN, ct, R, g) : find_gemm(false, id, dtype, scheme->R, g);
    if (!gemm) return fail(LCMA_ERR_NOKERNEL, "%s: no GEMM stage kernel for level %d fits the planes", who, level);

    // (the rows of the planes are the y dimension of the grids of Combine A and Combine H)
    if (g.bm / 16 > 65535) return fail(LCMA_ERR_SHAPE, "%s: M is too large", who);
    const int stages = tuning_unfused_stages(); // measurement aid: stages switched off keep the output of an earlier call
    // stage 1: Combine A (Eq. 3).  A takes the place of an N x K weight matrix in the Combine-B kernel
    // for that layout: block A_{i,l} is block (i, l), rows are k-contiguous.
    if (stages & 1) {
        PrepParams p;
        p.B = A;
        p.Bt = At;
        p.b_bytes = (uint32_t)(((M - 1) * lda + K) * es);
        p.bt_bytes = (uint32_t)((int64_t)R * g.bm * g.bk * es);
        p.ldb_b = (uint32_t)(lda * es);
        p.b_brow = (uint32_t)(g.bm * lda * es);
        p.b_bcol = (uint32_t)(g.bk * es);
        p.bt_ld_b = (uint32_t)(g.bk * es);
        p.bt_plane_b = (uint32_t)(g.bm * g.bk * es);
        p.bk = (int32_t)g.bk;
        p.bn = (int32_t)g.bm;
        p.n_row_b = (uint32_t)(K * es);
        const int64_t gy = (g.bk * es + 255) / 256;
        if (const int err = sk->launch_comb_a(&p, (int)(g.bm / 16), (int)gy, stream))
            return fail(LCMA_ERR_HIP, "%s: Combine-A launch failed with HIP error %d", who, err);
    }
    // stage 2: Combine B (Eq. 4), unless the planes of an earlier call are still valid (static weights)
    if (!reuse_bt && (stages & 2)) {
        const lcma_status st = prepare_b_planes(b_nk, N, K, B, ldb, dtype, scheme, Bt, stream, 128, es == 4 ? 16 : 64, sk);
        if (st != LCMA_OK) return st;
    }
    Params p;
    std::memset(&p, 0, sizeof p);
    p.alpha = 1.f;
    p.A = At;
    p.B = Bt;
    p.a_bytes = (uint32_t)((int64_t)R * g.bm * g.bk * es);
    p.b_bytes = (uint32_t)((int64_t)R * g.bn * g.bk * es);
    p.lda_b = p.ldb_b = (uint32_t)(g.bk * es);
    p.a_brow = (uint32_t)(g.bm * g.bk * es); // plane strides
    p.b_brow = (uint32_t)(g.bn * g.bk * es);
    p.nx = (int32_t)(g.bm / gemm->TM);
    p.nz = (int32_t)(g.bn / gemm->TN);
    p.ny = (int32_t)(g.bk / gemm->TK);
    p.k_row_b = (uint32_t)(Kp * es); // the planes are padded with zeros: no column of At is past K
    p.k_tail_b = (uint32_t)(g.bk * es);
    const int panel = tuning_panel();
    p.panel = panel < p.nz ? panel : p.nz;
    p.batch_order = tuning_batch_order(); // ablation: 1 = group-major
    if (level == 1) {
        // stage 3: the R products H_r = At_r x Bt_r as one batched launch of the plain kernel
        p.C = H;
        // 16-bit: the plane GEMM, which can hand the tile-products out in Split-Group ranges (Sec. 3.2) when the
        // workspace has room for the pieces beyond the planes; it writes the products in fp32 for fp16 storage.  The
        // generated batched kernel (ablations) writes them in fp16 for both 16-bit types.
        const bool planes = es == 2 && !forced_unfused_variant() && !p.batch_order;
        const int h_es = planes ? (int)g.h_es : es;
        p.c_bytes = (uint32_t)((int64_t)R * g.bm * g.bn * h_es);
        p.ldc_b = (uint32_t)(g.bn * h_es);
        p.c_brow = (uint32_t)(g.bm * g.bn * h_es);
        p.n_row_b = (uint32_t)(g.bn * h_es);
        if (!(stages & 4)) {
        } else if (planes) {
            PlaneGemmParams q;
            std::memset(&q, 0, sizeof q);
            q.A = At;
            q.B = Bt;
            q.C = H;
            q.a_bytes = p.a_bytes;
            q.b_bytes = p.b_bytes;
            q.c_bytes = p.c_bytes;
            q.lda_b = q.ldb_b = p.lda_b;
            q.ldc_b = p.ldc_b;
            q.a_plane = p.a_brow;
            q.b_plane = p.b_brow;
            q.c_plane = p.c_brow;
            q.ny = (int32_t)(g.bk * es / 128);
            q.n_row_b = p.n_row_b;
            if (const lcma_status st = plane_gemm(who, h_es == 4 ? PG_F16_F32 : PG_F16, q, R, g.bm, g.bn, 0, 0, H + g.h_bytes,
                                                  workspace_bytes - g.total(), stream))
                return st;
        } else {
            const int64_t grid = (int64_t)R * p.nx * p.nz;
            if (const int err = gemm->launch(&p, (int)grid, stream))
                return fail(LCMA_ERR_HIP, "%s: launch of %s failed with HIP error %d", who, gemm->name, err);
        }
        // stage 4: Combine H (Eq. 6)
        if (!(stages & 8)) return LCMA_OK;
        CombHParams h;
        h.H = H;
        h.C = C;
        h.h_bytes = p.c_bytes;
        h.c_bytes = (uint32_t)(((M - 1) * ldc + N) * es);
        h.h_ld_b = (uint32_t)(g.bn * h_es);
        h.h_plane_b = (uint32_t)(g.bm * g.bn * h_es);
        h.ldc_b = (uint32_t)(ldc * es);
        h.c_brow = (uint32_t)(g.bm * ldc * es);
        h.c_bcol = (uint32_t)(g.bn * es);
        h.n_row_b = (uint32_t)(N * es);
        const int64_t gy = (g.bn * es + 255) / 256;
        if (const int err = (h_es != es ? sk->launch_comb_h32 : sk->launch_comb_h)(&h, (int)(g.bm / 16), (int)gy, stream))
            return fail(LCMA_ERR_HIP, "%s: Combine-H launch failed with HIP error %d", who, err);
    } else {
        // stages 3 and 4 in one kernel: group by group, W applied to the fp32 accumulators
        p.C = C;
        p.c_bytes = (uint32_t)(((M - 1) * ldc + N) * es);
        p.ldc_b = (uint32_t)(ldc * es);
        p.c_brow = (uint32_t)(g.bm * ldc * es);
        p.c_bcol = (uint32_t)(g.bn * es);
        p.n_row_b = (uint32_t)(N * es);
        const int64_t grid = (int64_t)p.nx * p.nz;
        if (const int err = gemm->launch(&p, (int)grid, stream))
            return fail(LCMA_ERR_HIP, "%s: launch of %s failed with HIP error %d", who, gemm->name, err);
    }
    return LCMA_OK;
}
