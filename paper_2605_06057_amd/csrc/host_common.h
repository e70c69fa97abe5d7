// Host-side shared declarations of the LCMA library (not part of the public ABI).
#pragma once
#include <atomic>
#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/lcma.h"
#include "lcma_params.h"

struct lcma_scheme {
    int m = 0, k = 0, n = 0, R = 0;
    std::vector<int8_t> U, V, W; // R*m*k, R*k*n, R*m*n, row-major
    uint64_t hash = 0;
    int builtin = 0;                          // LCMA_STRASSEN.. when the coefficients are a built-in's, else 0
    mutable std::atomic<int> verified{0};     // 0 not checked, 1 Brent identity holds, 2 violated
    mutable int64_t first_bad = -1;
    mutable std::mutex mu;
};

namespace lcma {

// Records a thread-local message and returns `st`.
lcma_status fail(lcma_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

uint64_t scheme_hash(int m, int k, int n, int R, const int8_t *U, const int8_t *V, const int8_t *W);
const lcma_scheme *builtin_scheme(int id); // verified, cached; nullptr for LCMA_PLAIN / unknown
int builtin_id_of(const char *name);        // -1 if unknown
const char *builtin_name_of(int id);        // "plain" for LCMA_PLAIN; nullptr if unknown
int builtin_max_id();

// One generated kernel (scheme x dtype x tile x dataflow).
struct Variant {
    const char *name;
    int scheme_id;      // LCMA_PLAIN .. LCMA_LADERMAN
    int dtype;          // lcma_dtype
    int m, k, n, R;     // grid of the scheme it was generated for (1,1,1,1 for plain)
    uint64_t hash;      // scheme_hash of its coefficients (0 for plain)
    int TM, TN, TK;     // tile of one block product
    int chunk;          // products resident per pass (R: all H_r live, 1: Algorithm 2's r loop)
    int rank;           // >= 90: ablation variant, reachable by name only
    double eff;         // measured fraction of the dtype's MFMA peak its MFMA work sustains at large shapes
    int occ;            // work-groups per compute unit it is compiled for
    int products;       // block products it multiplies (R plus residual products)
    int prepared;       // 1: takes the output of the offline Combine-B kernel instead of B
    int b_nk;           // 1: takes B as the N x K weight matrix W (W[n][k] = B[k][n])
    int left_planes;    // 1: takes the output of the stand-alone Combine-A kernel instead of A (stage kernel)
    int batch;          // 1: batched plain GEMM over planes (stage kernel of the unfused dataflow)
    int (*launch)(const Params *p, int grid, void *stream); // returns a hipError_t
};
extern const Variant kVariants[];
extern const int kVariantCount;

// One generated offline Combine-B kernel (scheme x dtype).
struct PrepKernel {
    int scheme_id, dtype;
    int (*launch)(const PrepParams *p, int grid_x, int grid_y, void *stream);   // B given K x N; returns a hipError_t
    int (*launch_t)(const PrepParams *p, int grid_x, int grid_y, void *stream); // weights given N x K
};
extern const PrepKernel kPrepKernels[];
extern const int kPrepKernelCount;

// The stand-alone Combine-A and Combine-H kernels of one scheme x dtype (stages 1 and 4 of Algorithm 1).
struct StageKernel {
    int scheme_id, dtype;
    int planes; // planes every stage works on: R, or more when some products also have the rounding residual of their left
                // combination multiplied (a second plane pair with the W row of the product)
    int (*launch_comb_a)(const PrepParams *p, int grid_x, int grid_y, void *stream);
    // Combine B for `planes` planes, B given K x N / N x K; null when planes == R (the offline Combine-B kernels serve)
    int (*launch_comb_b)(const PrepParams *p, int grid_x, int grid_y, void *stream);
    int (*launch_comb_bt)(const PrepParams *p, int grid_x, int grid_y, void *stream);
    int (*launch_comb_h)(const CombHParams *p, int grid_x, int grid_y, void *stream);
    int (*launch_comb_h32)(const CombHParams *p, int grid_x, int grid_y, void *stream); // fp32 planes, 16-bit C; null for fp32 storage
    double rate_a, rate_b, rate_h; // measured algorithmic bytes per second of Combine A, Combine B, Combine H
};
extern const StageKernel kStageKernels[];
extern const int kStageKernelCount;

// The FP8 kernels of one scheme: Combine A and Combine B for N x K weights, each with the quantisation fused in.
struct Fp8Kernel {
    int scheme_id;
    int (*launch_comb_a)(const Fp8QuantParams *p, int grid_x, int grid_y, void *stream);
    int (*launch_prep_w)(const Fp8QuantParams *p, int grid_x, int grid_y, void *stream);
};
extern const Fp8Kernel kFp8Kernels[];
extern const int kFp8KernelCount;

// Offline Combine B into planes whose rows (N/n) and columns (K/k) are padded to multiples of n_gran / k_gran.
// stage (may be null): its Combine-B kernels and plane count take the place of the scheme's offline Combine-B kernels.
lcma_status prepare_b_planes(bool transposed, int64_t N, int64_t K, const void *B, int64_t ldb, lcma_dtype dtype,
                             const lcma_scheme *scheme, void *Bt, void *stream, int64_t n_gran, int64_t k_gran,
                             const StageKernel *stage = nullptr);

int dtype_size(int dtype); // bytes, or 0

// Measurement aids set by lcma_set_tuning (initial values: the LCMA_* environment variables, read once).
const Variant *forced_variant();
const Variant *forced_unfused_variant();
int tuning_panel();
int tuning_batch_order();

// The plane GEMM (csrc/lcma_plane_gemm.hpp, csrc/plane_gemm.cc): kinds of operand and output, scratch for the pieces of
// the Split-Group schedule, launch.
enum { PG_FP8_BF16 = 0, PG_FP8_F16 = 1, PG_F16 = 2, PG_BF16 = 3, PG_F16_OUT = 4 /* fp16 operands, fp16 C: same kernels as PG_F16 */,
       PG_F16_F32 = 5 /* fp16 operands, the fp32 sums stored as they are */ };
int64_t plane_gemm_scratch_bytes(int tile);
// predicted seconds of plane_gemm on `planes` planes of rows x cols with ny steps of 128 bytes (negative: no kernel fits)
double plane_gemm_seconds(int planes, int64_t rows, int64_t cols, int ny, int64_t scratch_bytes);
int64_t plane_gemm_static_steps(int64_t jobs, int ny, int tile);
int64_t plane_gemm_split_steps(int64_t jobs, int ny, int tile);
lcma_status plane_gemm(const char *who, int kind, PlaneGemmParams p, int planes, int64_t rows, int64_t cols, int tile,
                       int schedule, void *scratch, int64_t scratch_bytes, void *stream);
int tuning_schedule(); // 0 = choose, 1 = one tile-product per work-group, 2 = Split-Group ranges
int tuning_unfused_stages(); // bit 0 Combine A, bit 1 Combine B, bit 2 GEMM, bit 3 Combine H of lcma_gemm_unfused level 1

// C = beta * C for an M x N matrix (the product with K = 0), on `stream`.
lcma_status empty_product(int64_t M, int64_t N, void *C, int64_t ldc, int dtype, float beta, void *stream);

// The unfused dataflows on a workspace of `workspace_bytes` bytes (lcma_gemm_unfused and its variant on the
// library's static buffer); `who` names the entry point in messages.
lcma_status gemm_unfused(const char *who, int level, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                         const void *B, int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                         void *workspace, int64_t workspace_bytes, int reuse_bt, void *stream, bool b_nk = false);

// Variant of (scheme_id, dtype) with the smallest predicted time among those whose tile divides the
// shape; nullptr if none.
const Variant *pick_variant(int scheme_id, int dtype, int64_t M, int64_t N, int64_t K, int prepared = 0, int b_nk = 0);
// Predicted seconds of one variant on MI355X (MFMA time at its measured efficiency, stretched by
// wave quantisation on 256 compute units, bounded below by the compulsory HBM traffic, plus launch).
double predict_variant(const Variant &v, int64_t M, int64_t N, int64_t K);
bool variant_fits(const Variant &v, int64_t M, int64_t N, int64_t K);

} // namespace lcma

// hand-written auxiliary kernels (csrc/lcma_aux.hip); return a hipError_t
extern "C" int lcma_launch_range_flags_bf16(const void *X, int64_t rows, int64_t row_bytes, int64_t ld_bytes, void *flags, void *stream);
extern "C" int lcma_launch_scale_c(void *C, int64_t rows, int64_t row_bytes, int64_t ld_bytes, int dtype, float beta, void *stream);
extern "C" int lcma_launch_mfma_probe(const void *src, void *sink, int iters, void *stream);
