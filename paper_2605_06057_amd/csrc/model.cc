// Decision Module (paper Sec. 3.3) and the tile-scheduling arithmetic of Sec. 3.2.
//
// Two models live here.  lcma_model_stages / lcma_model_intensity are the paper's own
// formulas (Table 2, Eq. 8-10), kept so that they can be evaluated for any hardware tuple.
// lcma_predict_seconds is the model lcma_select uses for THIS library's kernels, whose
// combinations never travel through HBM: the cost of a scheme is then MFMA time (with wave
// quantisation on 256 compute units), vector-ALU time of the conversions and additions that
// are repeated by every work-group that stages a tile, and the compulsory HBM traffic.
#include "host_common.h"

#include <algorithm>
#include <cmath>

namespace lcma {

static const int kUnits = 256;           // compute units of MI355X
static const double kClock = 2.4e9;      // Hz
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

// Fraction of the MFMA peak that a kernel of this tile family sustains, and how much of the
// vector-ALU time fails to hide under it.  Measured on MI355X with this library's bench.
struct Calib {
    double eta_plain, eta_lcma, valu_exposed;
};
static Calib calib(int dtype) {
    if (dtype == LCMA_F32) return {0.60, 0.55, 0.5};
    return {0.45, 0.40, 0.5};
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
    const int es = dtype_size(dtype);
    if (!es || M <= 0 || N <= 0 || K <= 0) return -1.0;
    const Variant *v = pick_variant(scheme_id, dtype, M, N, K);
    if (!v) return -1.0;
    const Calib cal = calib(dtype);
    const double dM = (double)M, dN = (double)N, dK = (double)K;
    const double groups = (dM / (v->m * v->TM)) * (dN / (v->n * v->TN));
    const double waves = std::ceil(groups / kUnits);
    const double quant = waves * kUnits / groups; // idle share of the last wave
    const double eta = scheme_id == LCMA_PLAIN ? cal.eta_plain : cal.eta_lcma;
    const double t_mfma = 2.0 * dM * dN * dK * v->R / ((double)v->m * v->n * v->k) / (eta * mfma_peak(dtype)) * quant;
    double t_valu = 0.0;
    if (scheme_id != LCMA_PLAIN) {
        const lcma_scheme *s = builtin_scheme(scheme_id);
        if (!s) return -1.0;
        // lane-operations per element position of a staged tile: conversion of every raw tile
        // (bf16 only: 3 operations per packed pair) plus one addition per extra term.
        const double conv = dtype == LCMA_BF16 ? 1.5 : 0.0, add = es == 2 ? 0.5 : 1.0;
        // a chunked kernel re-stages raw tiles once per chunk that uses them
        const double passes = (double)v->R / v->chunk;
        const double rawA = std::min((double)nnz(s->U), passes * v->m * v->k);
        const double rawB = std::min((double)nnz(s->V), passes * v->k * v->n);
        const double a_ops = (conv * rawA + add * (nnz(s->U) - v->R)) * (dM / v->m) * (dK / v->k) * (dN / (v->n * v->TN));
        const double b_ops = (conv * rawB + add * (nnz(s->V) - v->R)) * (dK / v->k) * (dN / v->n) * (dM / (v->m * v->TM));
        const double c_ops = (double)nnz(s->W) * (dM / v->m) * (dN / v->n);
        t_valu = (a_ops + b_ops + c_ops) / (kUnits * 64.0 * kClock) * quant;
    }
    const double t_hbm = (dM * dK + dK * dN + dM * dN) * es / kHbmBytes;
    return std::max(t_hbm, t_mfma + cal.valu_exposed * t_valu) + kLaunch;
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
