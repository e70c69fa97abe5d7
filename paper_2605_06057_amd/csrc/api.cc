// C ABI entry points: argument checks, variant choice, kernel launch.
#include "host_common.h"

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

namespace lcma {

static thread_local char g_error[512] = "";

lcma_status fail(lcma_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return st;
}

// M is free (rows past M are padding the kernels never touch); N and K must keep rows 16-byte
// granular.
bool variant_fits(const Variant &v, int64_t M, int64_t N, int64_t K) {
    (void)M;
    (void)v;
    const int vec = 16 / dtype_size(v.dtype);
    return N % vec == 0 && K % vec == 0;
}
static bool fits(const Variant &v, int64_t M, int64_t N, int64_t K) { return variant_fits(v, M, N, K); }
static int64_t round_up(int64_t x, int64_t g) { return (x + g - 1) / g * g; }

const Variant *pick_variant(int scheme_id, int dtype, int64_t M, int64_t N, int64_t K, int prepared, int b_nk) {
    const Variant *best = nullptr;
    double best_t = 0.0;
    for (int i = 0; i < kVariantCount; ++i) {
        const Variant &v = kVariants[i];
        if (v.scheme_id != scheme_id || v.dtype != dtype || v.prepared != prepared || v.b_nk != b_nk || v.rank >= 90 || !fits(v, M, N, K))
            continue;
        const double t = predict_variant(v, M, N, K);
        if (!best || t < best_t) {
            best = &v;
            best_t = t;
        }
    }
    return best;
}

static const Variant *find_variant(const char *name) {
    for (int i = 0; i < kVariantCount; ++i)
        if (!std::strcmp(kVariants[i].name, name)) return &kVariants[i];
    return nullptr;
}

// Measurement aids (see lcma_set_tuning): process-wide, initialised once from the environment, never read from it again.
namespace {
std::atomic<const Variant *> g_forced{nullptr}, g_forced_unfused{nullptr};
std::atomic<int> g_panel{8}, g_batch_order{0}, g_schedule{0}, g_stages{15};
std::once_flag g_tuning_once;
bool set_tuning(const char *key, const char *value) {
    const char *v = value ? value : "";
    if (!std::strcmp(key, "variant")) g_forced = *v ? find_variant(v) : nullptr;
    else if (!std::strcmp(key, "unfused_variant")) g_forced_unfused = *v ? find_variant(v) : nullptr;
    else if (!std::strcmp(key, "panel")) g_panel = *v ? (std::atoi(v) < 1 ? 1 : std::atoi(v)) : 8;
    else if (!std::strcmp(key, "batch_order")) g_batch_order = *v ? std::atoi(v) != 0 : 0;
    else if (!std::strcmp(key, "schedule")) g_schedule = !std::strcmp(v, "static") ? 1 : !std::strcmp(v, "split") ? 2 : !std::strcmp(v, "persist") ? 3 : 0;
    else if (!std::strcmp(key, "unfused_stages")) g_stages = *v ? (std::atoi(v) & 15) : 15;
    else return false;
    return true;
}
void init_tuning() {
    std::call_once(g_tuning_once, [] {
        if (const char *e = std::getenv("LCMA_VARIANT")) set_tuning("variant", e);
        if (const char *e = std::getenv("LCMA_UNFUSED_VARIANT")) set_tuning("unfused_variant", e);
        if (const char *e = std::getenv("LCMA_PANEL")) set_tuning("panel", e);
        if (const char *e = std::getenv("LCMA_BATCH_ORDER")) set_tuning("batch_order", e);
        if (const char *e = std::getenv("LCMA_SCHEDULE")) set_tuning("schedule", e);
        if (const char *e = std::getenv("LCMA_UNFUSED_STAGES")) set_tuning("unfused_stages", e);
    });
}
} // namespace
const Variant *forced_variant() { init_tuning(); return g_forced.load(); }
const Variant *forced_unfused_variant() { init_tuning(); return g_forced_unfused.load(); }
int tuning_panel() { init_tuning(); return g_panel.load(); }
int tuning_batch_order() { init_tuning(); return g_batch_order.load(); }
int tuning_schedule() { init_tuning(); return g_schedule.load(); }
int tuning_unfused_stages() { init_tuning(); return g_stages.load(); }

// [p, p + bytes) and [q, q + qbytes) share a byte
static bool overlap(const void *p, int64_t bytes, const void *q, int64_t qbytes) {
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + (uintptr_t)qbytes && b < a + (uintptr_t)bytes;
}

// K = 0: the product of Eq. 1 is the zero matrix, so C = beta * C (zeros when beta is 0; C is then not read).
lcma_status empty_product(int64_t M, int64_t N, void *C, int64_t ldc, int dtype, float beta, void *stream) {
    const int es = dtype_size(dtype);
    if (!C) return fail(LCMA_ERR_ARG, "lcma_gemm: null matrix pointer");
    if (ldc < N) return fail(LCMA_ERR_ARG, "lcma_gemm: leading dimension smaller than the row");
    if (((uintptr_t)C & 15) || ((ldc * es) & 15) || N % (16 / es))
        return fail(LCMA_ERR_ARG, "lcma_gemm: C must be 16-byte aligned with rows of whole 16-byte vectors");
    if (((M - 1) * ldc + N) * es >= ((int64_t)1 << 31)) return fail(LCMA_ERR_SHAPE, "lcma_gemm: a matrix spans 2 GiB or more");
    if (const int err = lcma_launch_scale_c(C, M, N * es, ldc * es, dtype, beta, stream))
        return fail(LCMA_ERR_HIP, "lcma_gemm: launch failed with HIP error %d", err);
    return LCMA_OK;
}

// B and ldb describe the K x N matrix; for a variant that takes the weight layout, the N x K matrix W;
// for a prepared-B variant, the planes written by lcma_prepare_b (ldb is then ignored).
static lcma_status run(const Variant &v, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                       int64_t ldb, void *C, int64_t ldc, void *stream, float alpha = 1.f, float beta = 0.f) {
    const int es = dtype_size(v.dtype);
    if (v.left_planes || v.batch)
        return fail(LCMA_ERR_ARG, "lcma_gemm: %s is a stage kernel of lcma_gemm_unfused and takes no matrices", v.name);
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "lcma_gemm: negative size");
    if (M == 0 || N == 0) return LCMA_OK; // nothing to write
    if (K == 0) return empty_product(M, N, C, ldc, v.dtype, beta, stream);
    if (!A || !B || !C) return fail(LCMA_ERR_ARG, "lcma_gemm: null matrix pointer");
    if (v.prepared) ldb = N;
    if (lda < K || ldb < (v.b_nk ? K : N) || ldc < N)
        return fail(LCMA_ERR_ARG, "lcma_gemm: leading dimension smaller than the row");
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15)
        return fail(LCMA_ERR_ARG, "lcma_gemm: matrix pointers must be 16-byte aligned");
    if (((lda * es) | (ldb * es) | (ldc * es)) & 15)
        return fail(LCMA_ERR_ARG, "lcma_gemm: leading dimensions must be multiples of 16 bytes");
    if (!fits(v, M, N, K))
        return fail(LCMA_ERR_SHAPE, "lcma_gemm: N = %lld and K = %lld must be multiples of %d (16 bytes of elements)",
                    (long long)N, (long long)K, 16 / es);
    // blocks are cut from the matrices padded to whole tiles; the extents stay the true ones
    const int64_t Mp = round_up(M, (int64_t)v.m * v.TM), Np = round_up(N, (int64_t)v.n * v.TN),
                  Kp = round_up(K, (int64_t)v.k * v.TK);
    const int64_t bm = Mp / v.m, bn = Np / v.n, bk = Kp / v.k;
    const int64_t a_bytes = ((M - 1) * lda + K) * es,
                  b_bytes = v.prepared ? (int64_t)v.products * bn * bk * es
                            : v.b_nk   ? ((N - 1) * ldb + K) * es
                                       : ((K - 1) * ldb + N) * es,
                  c_bytes = ((M - 1) * ldc + N) * es;
    const int64_t lim = (int64_t)1 << 31;
    // offsets of padded rows and columns are formed in 32 bits before the range check drops them
    const int64_t b_span = v.b_nk ? (Np - 1) * ldb + Kp : (Kp - 1) * ldb + Np;
    if (((Mp - 1) * lda + Kp) * es >= lim || b_span * es >= lim || ((Mp - 1) * ldc + Np) * es >= lim ||
        b_bytes >= lim)
        return fail(LCMA_ERR_SHAPE, "lcma_gemm: a matrix spans 2 GiB or more");
    if (overlap(C, c_bytes, A, a_bytes) || overlap(C, c_bytes, B, b_bytes))
        return fail(LCMA_ERR_ARG, "lcma_gemm: C overlaps A or B");
    Params p;
    p.A = A;
    p.B = B;
    p.C = C;
    p.a_bytes = (uint32_t)a_bytes;
    p.b_bytes = (uint32_t)b_bytes;
    p.c_bytes = (uint32_t)c_bytes;
    p.lda_b = (uint32_t)(lda * es);
    p.ldb_b = (uint32_t)(ldb * es);
    p.ldc_b = (uint32_t)(ldc * es);
    p.a_brow = (uint32_t)(bm * lda * es);
    p.a_bcol = (uint32_t)(bk * es);
    p.b_brow = (uint32_t)(bk * ldb * es);
    p.b_bcol = (uint32_t)(bn * es);
    if (v.b_nk) { // block B_{l,j} is block (j, l) of W
        p.b_brow = (uint32_t)(bk * es);
        p.b_bcol = (uint32_t)(bn * ldb * es);
    }
    if (v.prepared) { // plane r: bn rows of bk elements
        p.ldb_b = (uint32_t)(bk * es);
        p.b_brow = (uint32_t)(bn * bk * es);
        p.b_bcol = 0;
    }
    p.c_brow = (uint32_t)(bm * ldc * es);
    p.c_bcol = (uint32_t)(bn * es);
    p.nx = (int32_t)(bm / v.TM);
    p.nz = (int32_t)(bn / v.TN);
    p.ny = (int32_t)(bk / v.TK);
    p.n_row_b = (uint32_t)(N * es);
    p.k_row_b = (uint32_t)(K * es);
    p.alpha = alpha;
    p.beta = beta;
    {   // first byte column inside the last block column of A whose tile reaches past K
        const int64_t valid = K - (int64_t)(v.k - 1) * bk; // columns of the last block inside K (may be <= 0)
        const int64_t whole = valid <= 0 ? 0 : valid / v.TK * v.TK;
        p.k_tail_b = (uint32_t)(whole * es);
    }
    const int64_t grid = (int64_t)p.nx * p.nz;
    if (grid >= lim) return fail(LCMA_ERR_SHAPE, "lcma_gemm: too many tiles");
    const int panel = tuning_panel();
    p.panel = panel < p.nz ? panel : p.nz;
    const int err = v.launch(&p, (int)grid, stream);
    if (err) return fail(LCMA_ERR_HIP, "lcma_gemm: launch of %s failed with HIP error %d", v.name, err);
    return LCMA_OK;
}

} // namespace lcma

using namespace lcma;

static lcma_status gemm(int b_nk, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                        void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme, void *stream, float alpha = 1.f,
                        float beta = 0.f) {
    if (!dtype_size(dtype)) return fail(LCMA_ERR_DTYPE, "lcma_gemm: unknown dtype %d", (int)dtype);
    int id = LCMA_PLAIN;
    if (scheme) {
        const lcma_status st = lcma_scheme_verify(scheme, nullptr);
        if (st != LCMA_OK) return st;
        id = scheme->builtin;
        if (!id)
            return fail(LCMA_ERR_NOKERNEL, "lcma_gemm: no kernel was generated for scheme <%d,%d,%d;%d> (hash %016llx)",
                        scheme->m, scheme->k, scheme->n, scheme->R, (unsigned long long)scheme->hash);
    }
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "lcma_gemm: negative size");
    if (M == 0 || N == 0) return LCMA_OK;
    const Variant *v = forced_variant(); // ablation override
    if (v && (v->scheme_id != id || v->dtype != (int)dtype || v->prepared || v->b_nk != b_nk)) v = nullptr;
    if (!v) v = pick_variant(id, dtype, M, N, K, 0, b_nk);
    if (!v) {
        bool any = false;
        for (int i = 0; i < kVariantCount; ++i)
            any |= kVariants[i].scheme_id == id && kVariants[i].dtype == (int)dtype && !kVariants[i].prepared &&
                   kVariants[i].b_nk == b_nk;
        if (!any)
            return fail(LCMA_ERR_NOKERNEL, "lcma_gemm: no kernel for scheme id %d with dtype %d%s", id, (int)dtype,
                        b_nk ? " that takes B as N x K" : "");
        return fail(LCMA_ERR_SHAPE, "lcma_gemm: no kernel of scheme id %d takes N = %lld (whole 16-byte vectors) and K = %lld (whole tiles)",
                    id, (long long)N, (long long)K);
    }
    return run(*v, M, N, K, A, lda, B, ldb, C, ldc, stream, alpha, beta);
}

extern "C" lcma_status lcma_gemm_ex(float alpha, float beta, int b_layout, int64_t M, int64_t N, int64_t K, const void *A,
                                    int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype,
                                    const lcma_scheme *scheme, void *stream) {
    if (b_layout != 0 && b_layout != 2)
        return fail(LCMA_ERR_ARG, "lcma_gemm_ex: b_layout must be 0 (B given K x N) or 2 (W given N x K)");
    if (!(alpha == alpha) || !(beta == beta)) return fail(LCMA_ERR_ARG, "lcma_gemm_ex: alpha or beta is not a number");
    return gemm(b_layout == 2, M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, stream, alpha, beta);
}

extern "C" lcma_status lcma_gemm(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                                 int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                                 void *stream) {
    return gemm(0, M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, stream);
}

extern "C" lcma_status lcma_gemm_nt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *W,
                                    int64_t ldw, void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                                    void *stream) {
    return gemm(1, M, N, K, A, lda, W, ldw, C, ldc, dtype, scheme, stream);
}

extern "C" lcma_status lcma_gemm_variant(const char *variant, int64_t M, int64_t N, int64_t K, const void *A,
                                         int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc, void *stream) {
    if (!variant) return fail(LCMA_ERR_ARG, "lcma_gemm_variant: null name");
    const Variant *v = find_variant(variant);
    if (!v) return fail(LCMA_ERR_NOKERNEL, "lcma_gemm_variant: no variant named '%s'", variant);
    return run(*v, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

static const PrepKernel *find_prep(int scheme_id, int dtype) {
    for (int i = 0; i < kPrepKernelCount; ++i)
        if (kPrepKernels[i].scheme_id == scheme_id && kPrepKernels[i].dtype == dtype) return &kPrepKernels[i];
    return nullptr;
}

// The prepared-B entry points need a verified scheme that kernels were generated for.
static lcma_status prepared_scheme(const lcma_scheme *scheme, const char *who, int *id) {
    if (!scheme) return fail(LCMA_ERR_ARG, "%s: a scheme is required", who);
    const lcma_status st = lcma_scheme_verify(scheme, nullptr);
    if (st != LCMA_OK) return st;
    if (!scheme->builtin)
        return fail(LCMA_ERR_NOKERNEL, "%s: no kernel was generated for scheme <%d,%d,%d;%d> (hash %016llx)", who,
                    scheme->m, scheme->k, scheme->n, scheme->R, (unsigned long long)scheme->hash);
    *id = scheme->builtin;
    return LCMA_OK;
}

extern "C" int64_t lcma_prepared_b_bytes(const lcma_scheme *scheme, int64_t N, int64_t K, lcma_dtype dtype) {
    const int es = dtype_size(dtype);
    if (!scheme || !es || N <= 0 || K <= 0 || N % (16 / es) || K % (16 / es)) return -1;
    return (int64_t)scheme->R * (round_up(N, (int64_t)scheme->n * 64) / scheme->n) *
           (round_up(K, (int64_t)scheme->k * (64 / es)) / scheme->k) * es;
}

namespace lcma {
// transposed: the input is the N x K weight matrix W (W[n][k] = B[k][n]) with leading dimension ldb.
// The planes hold N/n rows padded to a multiple of n_gran and K/k columns padded to a multiple of k_gran
// (multiples of 64 rows and 64 bytes).
lcma_status prepare_b_planes(bool transposed, int64_t N, int64_t K, const void *B, int64_t ldb, lcma_dtype dtype,
                             const lcma_scheme *scheme, void *Bt, void *stream, int64_t n_gran, int64_t k_gran,
                             const StageKernel *stage) {
    const char *who = transposed ? "lcma_prepare_bt" : "lcma_prepare_b";
    const int es = dtype_size(dtype);
    if (!es) return fail(LCMA_ERR_DTYPE, "%s: unknown dtype %d", who, (int)dtype);
    int id = 0;
    if (const lcma_status st = prepared_scheme(scheme, who, &id)) return st;
    const PrepKernel *pk = find_prep(id, dtype);
    const bool own = stage && stage->launch_comb_b; // the stage kernels bring their own Combine B (more planes than R)
    if (!pk && !own) return fail(LCMA_ERR_NOKERNEL, "%s: no Combine-B kernel for scheme id %d with dtype %d", who, id, (int)dtype);
    const int planes = own ? stage->planes : scheme->R;
    if (N < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (N == 0 || K == 0) return LCMA_OK;
    if (!B || !Bt) return fail(LCMA_ERR_ARG, "%s: null pointer", who);
    const int64_t rows = transposed ? N : K, cols = transposed ? K : N; // of the input as stored
    if (ldb < cols) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)B | (uintptr_t)Bt) & 15) || ((ldb * es) & 15))
        return fail(LCMA_ERR_ARG, "%s: pointers and the leading dimension must be multiples of 16 bytes", who);
    const int kt = 64 / es; // k granule of a plane
    if (N % (16 / es) || K % (16 / es))
        return fail(LCMA_ERR_SHAPE, "%s: N = %lld and K = %lld must be multiples of %d", who, (long long)N, (long long)K,
                    16 / es);
    // the planes hold the padded rows and columns (zeros)
    const int64_t bn = round_up(N, (int64_t)scheme->n * n_gran) / scheme->n,
                  bk = round_up(K, (int64_t)scheme->k * k_gran) / scheme->k;
    const int64_t b_bytes = ((rows - 1) * ldb + cols) * es, bt_bytes = (int64_t)planes * bn * bk * es;
    const int64_t lim = (int64_t)1 << 31;
    const int64_t prow = transposed ? bn * scheme->n : bk * scheme->k, pcol = transposed ? bk * scheme->k : bn * scheme->n;
    if (((prow - 1) * ldb + pcol) * es >= lim || bt_bytes >= lim)
        return fail(LCMA_ERR_SHAPE, "%s: a buffer spans 2 GiB or more", who);
    PrepParams p;
    p.B = B;
    p.Bt = Bt;
    p.b_bytes = (uint32_t)b_bytes;
    p.bt_bytes = (uint32_t)bt_bytes;
    p.ldb_b = (uint32_t)(ldb * es);
    p.bt_ld_b = (uint32_t)(bk * es);
    p.bt_plane_b = (uint32_t)(bn * bk * es);
    p.bk = (int32_t)bk;
    p.bn = (int32_t)bn;
    int gx, gy, err;
    if (transposed) {
        p.b_brow = (uint32_t)(bn * ldb * es); // from block row j of W to j + 1
        p.b_bcol = (uint32_t)(bk * es);       // from block column l of W to l + 1
        p.n_row_b = (uint32_t)(K * es);       // row length of W
        gx = (int)(bn / 16);
        gy = (int)((bk * es + 255) / 256);
        if (gx > 65535) return fail(LCMA_ERR_SHAPE, "%s: N is too large", who); // (the rows are the y dimension of the grid)
        err = (own ? stage->launch_comb_bt : pk->launch_t)(&p, gx, gy, stream);
    } else {
        p.b_brow = (uint32_t)(bk * ldb * es);
        p.b_bcol = (uint32_t)(bn * es);
        p.n_row_b = (uint32_t)(N * es);
        gx = (int)(bn / 64);
        gy = (int)(bk / kt);
        if (gx > 65535) return fail(LCMA_ERR_SHAPE, "%s: N is too large", who);
        err = (own ? stage->launch_comb_b : pk->launch)(&p, gx, gy, stream);
    }
    if (err) return fail(LCMA_ERR_HIP, "%s: launch failed with HIP error %d", who, err);
    return LCMA_OK;
}
} // namespace lcma

static lcma_status prepare_b(bool transposed, int64_t N, int64_t K, const void *B, int64_t ldb, lcma_dtype dtype,
                             const lcma_scheme *scheme, void *Bt, void *stream) {
    const int es = dtype_size(dtype); // 0 for an unknown dtype, which prepare_b_planes rejects first
    return prepare_b_planes(transposed, N, K, B, ldb, dtype, scheme, Bt, stream, 64, es ? 64 / es : 16);
}

extern "C" lcma_status lcma_prepare_b(int64_t N, int64_t K, const void *B, int64_t ldb, lcma_dtype dtype,
                                      const lcma_scheme *scheme, void *Bt, void *stream) {
    return prepare_b(false, N, K, B, ldb, dtype, scheme, Bt, stream);
}

extern "C" lcma_status lcma_prepare_bt(int64_t N, int64_t K, const void *W, int64_t ldw, lcma_dtype dtype,
                                       const lcma_scheme *scheme, void *Bt, void *stream) {
    return prepare_b(true, N, K, W, ldw, dtype, scheme, Bt, stream);
}

extern "C" lcma_status lcma_gemm_prepared(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *Bt,
                                          void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                                          void *stream) {
    if (!dtype_size(dtype)) return fail(LCMA_ERR_DTYPE, "lcma_gemm_prepared: unknown dtype %d", (int)dtype);
    int id = 0;
    if (const lcma_status st = prepared_scheme(scheme, "lcma_gemm_prepared", &id)) return st;
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "lcma_gemm_prepared: negative size");
    if (M == 0 || N == 0) return LCMA_OK;
    const Variant *v = forced_variant(); // ablation override
    if (v && (v->scheme_id != id || v->dtype != (int)dtype || !v->prepared)) v = nullptr;
    if (!v) v = pick_variant(id, dtype, M, N, K, 1);
    if (!v) {
        bool any = false;
        for (int i = 0; i < kVariantCount; ++i)
            any |= kVariants[i].scheme_id == id && kVariants[i].dtype == (int)dtype && kVariants[i].prepared;
        if (!any)
            return fail(LCMA_ERR_NOKERNEL, "lcma_gemm_prepared: no prepared-B kernel for scheme id %d with dtype %d", id,
                        (int)dtype);
        return fail(LCMA_ERR_SHAPE, "lcma_gemm_prepared: no kernel of scheme id %d takes N = %lld (whole 16-byte vectors) and K = %lld (whole tiles)",
                    id, (long long)N, (long long)K);
    }
    return run(*v, M, N, K, A, lda, Bt, N, C, ldc, stream);
}

extern "C" int lcma_variant_count(void) { return kVariantCount; }

extern "C" const char *lcma_variant_name(int index) {
    return (index >= 0 && index < kVariantCount) ? kVariants[index].name : nullptr;
}

extern "C" lcma_status lcma_variant_info(int index, int *scheme_id, int *dtype, int *TM, int *TN, int *TK, int *mult_M,
                                         int *mult_N, int *mult_K) {
    if (index < 0 || index >= kVariantCount) return fail(LCMA_ERR_ARG, "lcma_variant_info: index out of range");
    const Variant &v = kVariants[index];
    if (scheme_id) *scheme_id = v.scheme_id;
    if (dtype) *dtype = v.dtype;
    if (TM) *TM = v.TM;
    if (TN) *TN = v.TN;
    if (TK) *TK = v.TK;
    if (mult_M) *mult_M = v.m * v.TM;
    if (mult_N) *mult_N = v.n * v.TN;
    if (mult_K) *mult_K = v.k * v.TK;
    return LCMA_OK;
}

extern "C" const char *lcma_scheme_name(int scheme_id) { return builtin_name_of(scheme_id); }

extern "C" int lcma_scheme_id_max(void) { return builtin_max_id(); }

extern "C" int lcma_variant_prepared(int index) {
    return (index >= 0 && index < kVariantCount) ? kVariants[index].prepared : -1;
}

extern "C" int lcma_variant_b_layout(int index) {
    if (index < 0 || index >= kVariantCount) return -1;
    if (kVariants[index].left_planes || kVariants[index].batch) return 3;
    return kVariants[index].prepared ? 1 : kVariants[index].b_nk ? 2 : 0;
}

extern "C" const char *lcma_status_str(lcma_status st) {
    switch (st) {
    case LCMA_OK: return "ok";
    case LCMA_ERR_ARG: return "bad argument";
    case LCMA_ERR_IO: return "cannot read scheme";
    case LCMA_ERR_PARSE: return "malformed scheme text";
    case LCMA_ERR_BRENT: return "scheme violates the Brent equations";
    case LCMA_ERR_SHAPE: return "shape not supported by the tile";
    case LCMA_ERR_DTYPE: return "unknown dtype";
    case LCMA_ERR_NOKERNEL: return "no generated kernel";
    case LCMA_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

extern "C" const char *lcma_last_error(void) { return g_error; }

extern "C" lcma_status lcma_fp16_range_flags(int64_t rows, int64_t cols, const void *X, int64_t ld, void *flags, void *stream) {
    const char *who = "lcma_fp16_range_flags";
    if (rows < 0 || cols < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (!flags || ((uintptr_t)flags & 3)) return fail(LCMA_ERR_ARG, "%s: flags must be a 4-byte aligned device pointer", who);
    if (rows && cols) {
        if (!X || ((uintptr_t)X & 15) || ((ld * 2) & 15) || ld < cols) return fail(LCMA_ERR_ARG, "%s: X must be 16-byte aligned, ld a multiple of 8 and at least the row", who);
        if (cols % 8) return fail(LCMA_ERR_SHAPE, "%s: the row must be a multiple of 8 elements", who);
    }
    if (const int err = lcma_launch_range_flags_bf16(X, rows && cols ? rows : 0, cols * 2, ld * 2, flags, stream))
        return fail(LCMA_ERR_HIP, "%s: launch failed with HIP error %d", who, err);
    return LCMA_OK;
}

extern "C" lcma_status lcma_mfma_probe(const void *operands, void *sink, int64_t iters, double *flops, void *stream) {
    const char *who = "lcma_mfma_probe";
    if (!operands || !sink || ((uintptr_t)operands & 15) || ((uintptr_t)sink & 3))
        return fail(LCMA_ERR_ARG, "%s: operands (64 KiB, 16-byte aligned) and sink (2 MiB, 4-byte aligned) are required", who);
    if (iters < 1 || iters > 10000000) return fail(LCMA_ERR_ARG, "%s: iters must be between 1 and 10^7", who);
    if (flops) *flops = 2048.0 * 4.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
    if (const int err = lcma_launch_mfma_probe(operands, sink, (int)iters, stream))
        return fail(LCMA_ERR_HIP, "%s: launch failed with HIP error %d", who, err);
    return LCMA_OK;
}

extern "C" lcma_status lcma_set_tuning(const char *key, const char *value) {
    if (!key) return fail(LCMA_ERR_ARG, "lcma_set_tuning: null key");
    init_tuning();
    if (!set_tuning(key, value)) return fail(LCMA_ERR_ARG, "lcma_set_tuning: unknown key '%s'", key);
    return LCMA_OK;
}
