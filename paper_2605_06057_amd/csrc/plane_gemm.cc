// Host side of the plane GEMM (csrc/lcma_plane_gemm.hpp): choice of tile and of the schedule (Sec. 3.2, Split-Group
// Parallelism), launch.
#include "host_common.h"

#include <cstring>

#define LCMA_PG_DECL(NAME) extern "C" int lcma_launch_pg_##NAME(const lcma::PlaneGemmParams *p, void *stream);
LCMA_PG_DECL(fp8_t256_bf16)
LCMA_PG_DECL(fp8_t128_bf16)
LCMA_PG_DECL(fp8_t256_f16)
LCMA_PG_DECL(fp8_t128_f16)
LCMA_PG_DECL(f16_t256_f16)
LCMA_PG_DECL(f16_t128_f16)
LCMA_PG_DECL(f16_t256_f32)
LCMA_PG_DECL(f16_t128_f32)
LCMA_PG_DECL(bf16_t256_bf16)
LCMA_PG_DECL(bf16_t128_bf16)

namespace lcma {

namespace {
const int kCUs = 256;
typedef int (*Launch)(const PlaneGemmParams *, void *);
Launch launcher(int kind, int tile) {
    switch (kind * 2 + (tile == 256)) {
    case PG_FP8_BF16 * 2 + 1: return lcma_launch_pg_fp8_t256_bf16;
    case PG_FP8_BF16 * 2: return lcma_launch_pg_fp8_t128_bf16;
    case PG_FP8_F16 * 2 + 1: return lcma_launch_pg_fp8_t256_f16;
    case PG_FP8_F16 * 2: return lcma_launch_pg_fp8_t128_f16;
    case PG_F16 * 2 + 1: return lcma_launch_pg_f16_t256_f16;
    case PG_F16 * 2: return lcma_launch_pg_f16_t128_f16;
    case PG_BF16 * 2 + 1: return lcma_launch_pg_bf16_t256_bf16;
    case PG_BF16 * 2: return lcma_launch_pg_bf16_t128_bf16;
    case PG_F16_OUT * 2 + 1: return lcma_launch_pg_f16_t256_f16;
    case PG_F16_OUT * 2: return lcma_launch_pg_f16_t128_f16;
    case PG_F16_F32 * 2 + 1: return lcma_launch_pg_f16_t256_f32;
    case PG_F16_F32 * 2: return lcma_launch_pg_f16_t128_f32;
    }
    return nullptr;
}
int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
// work-groups that run at one time: one 256 x 256 tile (128 KB of LDS) or two 128 x 128 tiles (64 KB each) per CU
int slots_of(int tile) { return tile == 256 ? kCUs : 2 * kCUs; }
} // namespace

int64_t plane_gemm_scratch_bytes(int tile) { return (int64_t)slots_of(tile) * 2 * tile * tile * 4; }

// Steps (of 128 bytes of K) that the slowest work-group runs, for the time model: static launch in rounds of `slots`
// work-groups, Split-Group in one round of contiguous ranges.
int64_t plane_gemm_static_steps(int64_t jobs, int ny, int tile) { return ceil_div(jobs, slots_of(tile)) * ny; }
int64_t plane_gemm_split_steps(int64_t jobs, int ny, int tile) { return ceil_div(jobs * ny, slots_of(tile)); }

namespace {
// Tile and schedule together, by the steps the slowest work-group runs, in units of a step of the large tile.  A step of
// the small tile does a quarter of the work with two work-groups per CU, at three quarters of the efficiency
// (measured): 0.76 of a large step for two of them, so 0.38 each, twice as many run at once.  The Split-Group schedule
// adds the pieces: nearly every work-group holds two, 134 MB of fp32 partial sums in all, written at the end of the
// first kernel and read back by the second.  Measured against the other schedules on seven LLM shapes (plain, batched
// 16-bit and batched FP8 products): it wins only where it saves more than about 80 steps (few tile-products, long K:
// 64 tiles of K = 16384 run 26 % faster), and loses 3 to 25 % where the model had priced the pieces at 40.
// tile, schedule: 0 = choose.  Returns the cost in large steps (0 when nothing fits).
// What starting and finishing a tile-product costs, in steps of the large tile: a work-group of its own per tile-product
// (launch, first loads with nothing to overlap them, epilogue) against a persistent work-group that sends the first
// loads of its next tile-product during the last step of the current one (measured on the FFN shapes: the batched
// stage of Algorithm 1, 32 steps per tile-product, gains 9 %, the plain 16-bit product with 64 steps 2 to 4 %).  3.5
// fits both the 32-step tile-products of <2,2,2;7> (0.72 to 0.75 ms for 13 rounds) and the 16-step ones of <4,4,4;49>
// (0.74 ms for 22 rounds) at the FFN shape; what cannot be hidden is the tile of H_r a work-group writes out.
const double kTileCost = 5.0, kTileCostPersistent = 3.5;
// The Split-Group schedule adds the pieces (see below): as long as 80 steps of the large tile.
const double kSplitCost = 80.0;
// persist_ok: the persistent whole-tile schedule may be chosen (16-bit operands; the FP8 kernel loses 8 % with it: the
// scale bytes of the next tile-product are not fetched ahead)
double choose(int planes, int64_t rows, int64_t cols, int ny, int tile, int schedule, int64_t scratch_bytes, bool persist_ok,
              int *best_tile, int *best_sched) {
    double best = 0.0;
    *best_tile = *best_sched = 0;
    for (int t : {256, 128}) {
        if (tile && t != tile) continue;
        if (planes > 1 && (rows % t || cols % t)) continue; // planes lie back to back: a tile must not hang over the end of one
        const int64_t jobs = (int64_t)planes * ceil_div(rows, t) * ceil_div(cols, t);
        const double unit = t == 256 ? 1.0 : 0.76;
        for (int sc : {1, 2, 3}) {
            if (schedule ? sc != schedule : sc == 3 && !persist_ok) continue;
            if (sc == 2 && scratch_bytes < plane_gemm_scratch_bytes(t)) continue;
            // whole tile-products (one per work-group, or persistent work-groups that take every units-th one): rounds of
            // ny steps plus, per round, what starting and finishing a tile costs in steps; ranges of steps: one long round
            const double rounds = (double)ceil_div(jobs, slots_of(t));
            const double steps = sc == 2 ? (double)plane_gemm_split_steps(jobs, ny, t) + kSplitCost
                                         : rounds * (ny + (sc == 3 && rounds > 1 ? kTileCostPersistent : kTileCost));
            const double cost = steps * unit * (sc == 2 ? 1.05 : 1.0); // the persistent kernel's step is 5 % slower
            if (!*best_tile || cost < best) {
                best = cost;
                *best_tile = t;
                *best_sched = sc;
            }
        }
    }
    return best;
}
} // namespace

// Seconds of a plane GEMM for the time model (Sec. 3.3): the steps of the slowest work-group under the tile and schedule
// that plane_gemm would choose, at the time of a step of the 256 x 256 tile measured on the FFN shapes with random
// operands (1.62 us for 16-bit and for FP8 operands: a step is 128 bytes of K either way and both run into the
// chip's power limit), plus a fixed 8 us for every tile a work-group works through (launch, first loads, epilogue).
double plane_gemm_seconds(int planes, int64_t rows, int64_t cols, int ny, int64_t scratch_bytes) {
    int t = 0, sc = 0;
    const double steps = choose(planes, rows, cols, ny, 0, tuning_schedule(), scratch_bytes, true, &t, &sc);
    if (!t) return -1.0;
    return steps * 1.62e-6;
}

// p: operands, extents, pitches, plane strides, ny, n_row_b filled in by the caller for `planes` planes of rows x cols
// (padded sizes, multiples of the tile when batched).  tile: 256 or 128, 0 = choose.  schedule: 0 = choose, 1 = one
// tile-product per work-group, 2 = Split-Group ranges (needs `scratch` of plane_gemm_scratch_bytes(tile) bytes), 3 =
// persistent work-groups that each take every units-th whole tile-product.
lcma_status plane_gemm(const char *who, int kind, PlaneGemmParams p, int planes, int64_t rows, int64_t cols, int tile,
                       int schedule, void *scratch, int64_t scratch_bytes, void *stream) {
    const int forced = tuning_schedule();
    if (forced) schedule = forced;
    int best_tile = 0, best_sched = 0;
    choose(planes, rows, cols, p.ny, tile, schedule, scratch ? scratch_bytes : 0, kind != PG_FP8_BF16 && kind != PG_FP8_F16, &best_tile,
           &best_sched);
    if (!best_tile) {
        if (schedule == 2)
            return fail(LCMA_ERR_ARG, "%s: the Split-Group schedule needs %lld bytes of scratch", who,
                        (long long)plane_gemm_scratch_bytes(tile ? tile : 256));
        return fail(LCMA_ERR_SHAPE, "%s: planes must be whole tiles", who);
    }
    tile = best_tile;
    schedule = best_sched;
    Launch launch = launcher(kind, tile);
    if (!launch) return fail(LCMA_ERR_NOKERNEL, "%s: no plane GEMM kernel of kind %d", who, kind);
    p.nx = (int32_t)ceil_div(rows, tile);
    p.nz = (int32_t)ceil_div(cols, tile);
    const int64_t jobs = (int64_t)planes * p.nx * p.nz, total = jobs * p.ny;
    if (total >= ((int64_t)1 << 31)) return fail(LCMA_ERR_SHAPE, "%s: too many tile steps", who);
    p.jobs = (int32_t)jobs;
    // column panels of the tile order: 8 tiles wide, or the widest of 7, 6, 5 that leaves no narrower panel at the end
    // (28 columns of tiles as 4 x 7 instead of 3 x 8 + 4: the batched stage at the FFN shape 1 % faster)
    int panel = tuning_panel();
    if (panel == 8 && p.nz % 8)
        for (int w : {7, 6, 5})
            if (p.nz % w == 0) {
                panel = w;
                break;
            }
    p.panel = panel < p.nz ? panel : p.nz;
    const int slots = slots_of(tile);
    p.interleave = 0;
    if (schedule == 3) { // persistent work-groups, whole tile-products u, u + units, ...
        p.units = (int32_t)(jobs < slots ? jobs : slots);
        p.cap = p.ny;
        // batches of planes: rounds of consecutive tile-products; one product: an eighth of them per XCD (see
        // PlaneGemm::run), which needs the same number of work-groups on every XCD (with fewer tile-products than slots
        // units == jobs and the launcher takes the kernel with a work-group per tile-product anyway)
        p.interleave = planes > 1 || (p.units & 7) ? 1 : 2;
        p.partial = nullptr;
    } else if (schedule == 2) {
        p.units = (int32_t)(total < slots ? total : slots);
        p.cap = ceil_div(total, p.units);
        p.units = (int32_t)ceil_div(total, p.cap); // no idle work-group at the end
        p.partial = scratch;
    } else {
        p.units = (int32_t)jobs;
        p.cap = p.ny;
        p.partial = nullptr;
    }
    if (const int err = launch(&p, stream)) return fail(LCMA_ERR_HIP, "%s: plane GEMM launch failed with HIP error %d", who, err);
    return LCMA_OK;
}

} // namespace lcma

using namespace lcma;

// Plain GEMM for weights stored N x K on the plane GEMM, with a workspace that lets it split tile-products between
// work-groups (see include/lcma.h).
extern "C" lcma_status lcma_gemm_nt_ws(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *W, int64_t ldw,
                                       void *C, int64_t ldc, lcma_dtype dtype, void *workspace, int64_t workspace_bytes,
                                       void *stream) {
    const char *who = "lcma_gemm_nt_ws";
    if (dtype != LCMA_BF16 && dtype != LCMA_F16) {
        if (!dtype_size(dtype)) return fail(LCMA_ERR_DTYPE, "%s: unknown dtype %d", who, (int)dtype);
        return lcma_gemm_nt(M, N, K, A, lda, W, ldw, C, ldc, dtype, nullptr, stream);
    }
    if (M < 0 || N < 0 || K < 0) return fail(LCMA_ERR_ARG, "%s: negative size", who);
    if (M == 0 || N == 0) return LCMA_OK;
    if (K == 0 || K % 64) return lcma_gemm_nt(M, N, K, A, lda, W, ldw, C, ldc, dtype, nullptr, stream); // steps of 64 elements
    if (!A || !W || !C) return fail(LCMA_ERR_ARG, "%s: null matrix pointer", who);
    if (lda < K || ldw < K || ldc < N) return fail(LCMA_ERR_ARG, "%s: leading dimension smaller than the row", who);
    if ((((uintptr_t)A | (uintptr_t)W | (uintptr_t)C) & 15) || (((lda | ldw | ldc) * 2) & 15))
        return fail(LCMA_ERR_ARG, "%s: pointers and leading dimensions must be multiples of 16 bytes", who);
    if (N % 8) return fail(LCMA_ERR_SHAPE, "%s: N = %lld must be a multiple of 8", who, (long long)N);
    const int64_t lim = (int64_t)1 << 31, Mp = (M + 255) / 256 * 256, Np = (N + 255) / 256 * 256;
    if (((Mp - 1) * lda + K) * 2 >= lim || ((Np - 1) * ldw + K) * 2 >= lim || ((Mp - 1) * ldc + Np) * 2 >= lim)
        return fail(LCMA_ERR_SHAPE, "%s: a matrix spans 2 GiB or more", who);
    PlaneGemmParams p;
    std::memset(&p, 0, sizeof p);
    p.A = A;
    p.B = W;
    p.C = C;
    p.a_bytes = (uint32_t)(((M - 1) * lda + K) * 2);
    p.b_bytes = (uint32_t)(((N - 1) * ldw + K) * 2);
    p.c_bytes = (uint32_t)(((M - 1) * ldc + N) * 2);
    p.lda_b = (uint32_t)(lda * 2);
    p.ldb_b = (uint32_t)(ldw * 2);
    p.ldc_b = (uint32_t)(ldc * 2);
    p.ny = (int32_t)(K / 64);
    p.n_row_b = (uint32_t)(N * 2);
    if (workspace && ((uintptr_t)workspace & 255)) return fail(LCMA_ERR_ARG, "%s: the workspace must be 256-byte aligned", who);
    return plane_gemm(who, dtype == LCMA_BF16 ? PG_BF16 : PG_F16_OUT, p, 1, M, N, 0, 0, workspace, workspace ? workspace_bytes : 0, stream);
}
