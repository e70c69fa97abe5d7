// Decision Module (paper Sec. 3.3) and the tile-scheduling arithmetic of Sec. 3.2.
//
// Two models live here.  lcma_model_stages / lcma_model_intensity are the paper's own
// formulas (Table 2, Eq. 8-10), kept so that they can be evaluated for any hardware tuple.
// lcma_predict_seconds is the model lcma_select uses for THIS library's kernels, whose
// combinations never travel through HBM, so the paper's memory terms do not apply.  What the
// additions, conversions and LDS traffic of a fused kernel cost shows in the fraction of the
// MFMA peak that kernel sustains; that fraction is measured once per generated kernel and kept
// in the kernel table.  A prediction is then MFMA time at that efficiency, stretched by wave
// quantisation on 256 compute units and bounded below by the compulsory HBM traffic.
#include "host_common.h"

#include <algorithm>
#include <cmath>

namespace lcma {

static const int kUnits = 256;           // compute units of MI355X
static const double kHbmBytes = 8.0e12;  // bytes/s
static const double kLaunch = 4.0e-6;    // seconds per launch

int dtype_size(int dtype) {
    switch (dtype) {
    case LCMA_F32: return 4;
    case LCMA_BF16:
    case LCMA_F16: return 2;
    default: return 0;
    }
}

static double mfma_peak(int dtype) { return dtype == LCMA_F32 ? 157.3e12 : 2516.6e12; }

static int nnz(const std::vector<int8_t> &v) {
    int c = 0;
    for (int8_t x : v) c += x != 0;
    return c;
}

double predict_variant(const Variant &v, int64_t M, int64_t N, int64_t K) {
    const int es = dtype_size(v.dtype);
    // padded to whole tiles, as the kernels run them
    const double dM = std::ceil((double)M / (v.m * v.TM)) * (v.m * v.TM),
                 dN = std::ceil((double)N / (v.n * v.TN)) * (v.n * v.TN), dK = (double)K;
    const double groups = (dM / (v.m * v.TM)) * (dN / (v.n * v.TN));
    // Work-groups run in rounds of 256 * occ.  A round that leaves every CU with a single work-group
    // of a kernel built for two per CU is shorter than a full one: alone, a work-group takes ~0.63 of
    // the time it takes beside a neighbour (measured on the plain and Strassen kernels).
    const double slots = (double)kUnits * v.occ;
    const double t_round = slots * (2.0 * v.TM * v.TN * dK * v.products / v.k) / (v.eff * mfma_peak(v.dtype));
    const double full = std::floor(groups / slots), rest = groups - full * slots;
    double rounds = full;
    if (rest > 0) rounds += (v.occ > 1 && rest <= kUnits) ? 0.63 : 1.0;
    const double t_mfma = rounds * t_round;
    const double t_hbm = (dM * dK + dK * dN + dM * dN) * es / kHbmBytes;
    return std::max(t_hbm, t_mfma) + kLaunch;
}

} // namespace lcma

using namespace lcma;

extern "C" lcma_status lcma_hw_mi355x(lcma_dtype dtype, lcma_hw *out) {
    const int es = dtype_size(dtype);
    if (!es) return fail(LCMA_ERR_DTYPE, "lcma_hw_mi355x: unknown dtype %d", (int)dtype);
    if (!out) return fail(LCMA_ERR_ARG, "lcma_hw_mi355x: null output");
    out->flops_mul = mfma_peak(dtype);
    // additions per second: the fp32 vector rate counts a fused multiply-add as two operations;
    // 16-bit additions run two per lane.
    out->flops_add = (es == 4) ? 78.65e12 : 157.3e12;
    out->beta = kHbmBytes / es;
    return LCMA_OK;
}

extern "C" lcma_status lcma_model_stages(const lcma_scheme *s, int64_t M, int64_t N, int64_t K, const lcma_hw *hw,
                                         lcma_stage_costs *out) {
    if (!hw || !out || M <= 0 || N <= 0 || K <= 0) return fail(LCMA_ERR_ARG, "lcma_model_stages: bad argument");
    const double dM = (double)M, dN = (double)N, dK = (double)K;
    for (int i = 0; i < 4; ++i) out->flops[i] = out->elems[i] = out->seconds[i] = 0.0;
    if (!s) { // Table 2, first row
        out->flops[2] = 2.0 * dM * dN * dK;
        out->elems[2] = dM * dK + dN * dK + dM * dN;
        out->seconds[2] = std::max(out->flops[2] / hw->flops_mul, out->elems[2] / hw->beta);
        return LCMA_OK;
    }
    const double m = s->m, k = s->k, n = s->n, R = s->R;
    const double nu = nnz(s->U), nv = nnz(s->V), nw = nnz(s->W);
    out->flops[0] = (nu - R) * (dM / m) * (dK / k);
    out->elems[0] = dM * dK * (1.0 + R / (m * k));
    out->flops[1] = (nv - R) * (dN / n) * (dK / k);
    out->elems[1] = dN * dK * (1.0 + R / (n * k));
    out->flops[2] = 2.0 * R * dM * dN * dK / (m * n * k);
    out->elems[2] = R * (dM * dK / (m * k) + dN * dK / (n * k) + dM * dN / (m * n));
    out->flops[3] = (nw - m * n) * (dM / m) * (dN / n);
    out->elems[3] = dM * dN * (1.0 + R / (m * n));
    for (int i = 0; i < 4; ++i) {
        const double rate = (i == 2) ? hw->flops_mul : hw->flops_add;
        out->seconds[i] = std::max(out->flops[i] / rate, out->elems[i] / hw->beta);
    }
    return LCMA_OK;
}

extern "C" lcma_status lcma_model_intensity(const lcma_scheme *s, int64_t M, int64_t N, int64_t K, double *eq8,
                                            double *eq9, double *eq10) {
    if (M <= 0 || N <= 0 || K <= 0) return fail(LCMA_ERR_ARG, "lcma_model_intensity: bad shape");
    const double dM = (double)M, dN = (double)N, dK = (double)K;
    const double mnk2 = 2.0 * dM * dN * dK;
    if (eq8) *eq8 = mnk2 / (dM * dK + dN * dK + dM * dN);
    if (s) {
        const double m = s->m, k = s->k, n = s->n, R = s->R;
        const double gain = mnk2 * (1.0 - R / (m * n * k));
        const double ab = dM * dK * (1.0 + R / (m * k)) + dN * dK * (1.0 + R / (n * k));
        if (eq9) *eq9 = gain / (ab + dM * dN * (1.0 + R / (m * n)));
        if (eq10) *eq10 = gain / (ab + dM * dN);
    } else {
        if (eq9) *eq9 = 0.0;
        if (eq10) *eq10 = 0.0;
    }
    return LCMA_OK;
}

extern "C" double lcma_predict_seconds(int scheme_id, int64_t M, int64_t N, int64_t K, lcma_dtype dtype) {
    if (!dtype_size(dtype) || M <= 0 || N <= 0 || K <= 0) return -1.0;
    const Variant *v = pick_variant(scheme_id, dtype, M, N, K);
    return v ? predict_variant(*v, M, N, K) : -1.0;
}

extern "C" int lcma_select(int64_t M, int64_t N, int64_t K, lcma_dtype dtype) {
    const int es = dtype_size(dtype);
    if (!es || M <= 0 || N <= 0 || K <= 0) return -1;
    // Eq. 8: a GEMM that is already memory-bound cannot gain from fewer multiplications.
    lcma_hw hw;
    lcma_hw_mi355x(dtype, &hw);
    double ai = 0.0;
    lcma_model_intensity(nullptr, M, N, K, &ai, nullptr, nullptr);
    if (ai <= hw.flops_mul / hw.beta) return LCMA_PLAIN;
    int best = LCMA_PLAIN;
    double best_t = lcma_predict_seconds(LCMA_PLAIN, M, N, K, dtype);
    for (int id = LCMA_STRASSEN; id <= LCMA_LADERMAN; ++id) {
        const double t = lcma_predict_seconds(id, M, N, K, dtype);
        if (t > 0.0 && (best_t <= 0.0 || t < best_t)) {
            best = id;
            best_t = t;
        }
    }
    return best;
}

extern "C" lcma_status lcma_sched_waves(int64_t groups, int R, int units, int64_t *tile_level, int64_t *group_level) {
    if (groups < 0 || R <= 0 || units <= 0) return fail(LCMA_ERR_ARG, "lcma_sched_waves: bad argument");
    if (tile_level) *tile_level = (groups * R + units - 1) / units;
    if (group_level) *group_level = ((groups + units - 1) / units) * R;
    return LCMA_OK;
}

extern "C" lcma_status lcma_sched_range(int64_t groups, int R, int units, int unit, int64_t *begin, int64_t *end) {
    if (groups < 0 || R <= 0 || units <= 0 || unit < 0 || unit >= units || !begin || !end)
        return fail(LCMA_ERR_ARG, "lcma_sched_range: bad argument");
    const int64_t total = groups * R;
    const int64_t cap = (total + units - 1) / units;
    *begin = std::min(total, cap * unit);
    *end = std::min(total, cap * (unit + 1));
    return LCMA_OK;
}
