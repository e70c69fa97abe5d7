/*
 * lcma.h - C ABI of the MI355X (gfx950) lower-complexity matrix multiplication library.
 *
 * The library computes C = A x B (paper Eq. 1) either with a plain MFMA GEMM or with
 * an LCMA, a bilinear scheme L = <m,k,n,R,U,V,W> (paper Sec. 2.1): A, B and C are cut
 * into m x k, k x n and m x n grids of blocks, R operand combinations are formed
 * (Eq. 3, Eq. 4), R block products are taken (Eq. 5) and combined into the blocks of C
 * (Eq. 6).  On the GPU the four stages run as ONE launch: combinations are formed on
 * chip while tiles are staged, the R products of a group (Sec. 3.2, Group-Parallel
 * Optimization) stay in registers and W is applied in fp32 before one final rounding.
 *
 * General conventions
 *   - Matrices are row-major, never transposed; ld* are in ELEMENTS (not bytes).
 *   - A, B, C are DEVICE pointers owned by the caller; the library neither keeps nor
 *     frees them; C must not overlap A or B (checked: ARG).  lcma_gemm and lcma_gemm_nt overwrite C;
 *     lcma_gemm_ex adds the usual alpha / beta scaling.  K = 0 is the empty product: C = beta * C, zeros for
 *     the calls without beta.
 *   - Scheme handles and everything else are HOST objects.
 *   - No function aborts or throws; every failure is a status code, and
 *     lcma_last_error() returns a thread-local description of the latest one.
 */
#ifndef LCMA_H
#define LCMA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LCMA_OK = 0,
    LCMA_ERR_ARG = 1,      /* null pointer, negative size, misaligned pointer or ld  */
    LCMA_ERR_IO = 2,       /* scheme file cannot be read                              */
    LCMA_ERR_PARSE = 3,    /* scheme text is malformed                                */
    LCMA_ERR_BRENT = 4,    /* coefficients do not multiply matrices                   */
    LCMA_ERR_SHAPE = 5,    /* N or K not a whole number of 16-byte vectors, or a matrix of 2 GiB or more */
    LCMA_ERR_DTYPE = 6,    /* unknown dtype                                           */
    LCMA_ERR_NOKERNEL = 7, /* no kernel was generated for this scheme / dtype         */
    LCMA_ERR_HIP = 8       /* the HIP runtime reported an error                       */
} lcma_status;

/* Storage type of A, B and C.  Accumulation is always fp32. */
typedef enum { LCMA_F32 = 0, LCMA_BF16 = 1, LCMA_F16 = 2 } lcma_dtype;

/* Built-in scheme ids, also the return values of lcma_select. */
enum { LCMA_PLAIN = 0, LCMA_STRASSEN = 1, LCMA_STRASSEN2 = 2, LCMA_LADERMAN = 3 };

typedef struct lcma_scheme lcma_scheme; /* opaque, immutable once loaded */

/* ------------------------------------------------------------------ schemes (Sec. 2.1)
 * lcma_scheme_load: `spec` is "builtin:strassen" (<2,2,2;7>), "builtin:strassen2"
 * (<4,4,4;49>, the Kronecker square of Strassen), "builtin:laderman" (<3,3,3;23>), or
 * the path of a text file: first line `m k n R`, then R lines of m*k integers (U[r],
 * row-major over (i,l)), R lines of k*n integers (V[r] over (l,j)), R lines of m*n
 * integers (W[r] over (i,j)); '#' starts a comment; coefficients must fit in int8.
 * On success *out owns a new handle (release with lcma_scheme_free).  The handle is
 * NOT yet verified.  Errors: ARG, IO, PARSE.
 */
lcma_status lcma_scheme_load(const char *spec, lcma_scheme **out);

/* lcma_scheme_verify: exact integer check of the Brent identity
 *   sum_r U[r,i,a] V[r,b,j] W[r,c,d] == [a==b][i==c][j==d]
 * (Eq. 3-5 substituted into Eq. 6, coefficient of A_{i,a}B_{b,j} in C_{c,d}).
 * Returns LCMA_OK or LCMA_ERR_BRENT; when first_bad is not NULL it receives the flat
 * row-major index over (i,a,b,j,c,d), extents (m,k,k,n,m,n), of the first violated
 * equation, or -1.  The verdict is cached in the handle (thread-safe).
 */
lcma_status lcma_scheme_verify(const lcma_scheme *s, int64_t *first_bad);

void lcma_scheme_free(lcma_scheme *s);

/* Grid, rank and the non-zero counts ||U||_0, ||V||_0, ||W||_0 (any pointer may be NULL). */
lcma_status lcma_scheme_info(const lcma_scheme *s, int *m, int *k, int *n, int *R,
                             int *nnzU, int *nnzV, int *nnzW);

/* Copies the coefficients out: U holds R*m*k, V R*k*n, W R*m*n int8 values (host memory). */
lcma_status lcma_scheme_coeffs(const lcma_scheme *s, int8_t *U, int8_t *V, int8_t *W);

/* ------------------------------------------------------------------ the GEMM (Eq. 1, Eq. 3-6, Algorithm 2)
 * lcma_gemm: C[M x N] = A[M x K] x B[K x N] on the current device, asynchronously on
 * `stream` (a hipStream_t; NULL = the default stream).  `dtype` is the storage type of
 * all three matrices.  scheme == NULL runs the plain MFMA GEMM; otherwise the scheme
 * must pass lcma_scheme_verify (run and cached on first use) and have a generated
 * kernel.  Shapes: M is free; N and K must be multiples of 16 bytes of elements (8 for the
 * 16-bit types, 4 for F32).  The blocks of the scheme (the paper takes ceil(M/m) x
 * ceil(K/k) etc., Sec. 2.1) are cut from the matrices padded with zero rows and columns
 * to whole tiles; the padding is never read from or written to memory.
 * Pointers must be 16-byte aligned and lda, ldb, ldc multiples of 16 bytes; each
 * matrix, padded to whole tiles, must span less than 2 GiB.  With 16-bit inputs the combinations of Eq. 3/4 are
 * formed and multiplied in fp16 (bf16 inputs are converted exactly for |x| in
 * [2^-14, 65504]; larger magnitudes overflow, smaller ones lose bits); H_r (Eq. 5) and
 * the W-combination (Eq. 6) stay in fp32 and C is rounded once.
 * Errors: ARG, BRENT, SHAPE, DTYPE, NOKERNEL, HIP.  Nothing is launched on error.
 */
lcma_status lcma_gemm(int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb,
                      void *C, int64_t ldc, lcma_dtype dtype,
                      const lcma_scheme *scheme, void *stream);

/* Range guard for BF16 storage.  The LCMA kernels (every scheme != NULL, and lcma_gemm_unfused) convert bf16 inputs to
 * fp16, form the combinations of Eq. 3 / Eq. 4 and multiply in fp16.  That is exact for magnitudes in [2^-14, 32752];
 * outside it: a magnitude above 65504 is replaced by 65504 (the conversion rounds toward zero), a two-term sum of values
 * above 32752 can reach fp16 infinity (C then holds Inf or NaN), and a non-zero magnitude below 2^-14 lands in fp16's
 * subnormal range and loses low bits (below 2^-24: becomes zero).  Nothing is signalled.  The plain GEMM (scheme ==
 * NULL) multiplies bf16 as it is and has no such limit, and the FP8 path scales per block.  A caller that cannot vouch
 * for the range runs this check (once for static weights) and takes the plain GEMM when a flag comes back:
 * lcma_fp16_range_flags writes to the device word *flags (asynchronously on `stream`): bit 0 = some |x| > 32752 (or Inf /
 * NaN), bit 1 = some 0 < |x| < 2^-14.  X: rows x cols bf16, ld in elements (multiple of 8), 16-byte aligned, cols a
 * multiple of 8.  One pass over X at memory speed.  Errors: ARG, SHAPE, HIP. */
lcma_status lcma_fp16_range_flags(int64_t rows, int64_t cols, const void *X, int64_t ld, void *flags, void *stream);

/* Measurement aid, not part of the path: what the matrix pipe sustains on given operand VALUES with no memory traffic at
 * all (the 16-bit roofline of a power-limited chip: MI355X runs dense fp16 / bf16 products of random values well below
 * the rate it reaches on zeros).  2048 work-groups of four waves; every wave takes eight fragments from `operands`
 * (device, 64 KiB = 4096 vectors of eight fp16 values, 16-byte aligned, read only) and runs `iters` (1 .. 10^7) rounds of
 * eight independent 32x32x16 fp16 MFMA instructions; one float per thread goes to `sink` (device, 2 MiB, overwritten).
 * *flops (host, may be NULL) receives the floating-point operations of the launch, 2048 * 4 * iters * 8 * 32768; the
 * caller times the launch.  Asynchronous on `stream`.  Errors: ARG, HIP. */
lcma_status lcma_mfma_probe(const void *operands, void *sink, int64_t iters, double *flops, void *stream);

/* lcma_gemm with the right operand given the way a linear layer stores its weight (the operand the
 * paper's end-to-end evaluation multiplies by): W is N x K row-major, ldw in elements, and
 * C[M x N] = A[M x K] x W^T, that is B[k][n] = W[n][k] in Eq. 1.  Everything else (types, sizes,
 * alignment, padding, arithmetic, errors) is lcma_gemm's; the result is the same bit for bit.
 * NOKERNEL when no kernel taking this layout was generated for the scheme and dtype. */
lcma_status lcma_gemm_nt(int64_t M, int64_t N, int64_t K,
                         const void *A, int64_t lda, const void *W, int64_t ldw,
                         void *C, int64_t ldc, lcma_dtype dtype,
                         const lcma_scheme *scheme, void *stream);

/* lcma_gemm with the usual scaling of a GEMM interface (Eq. 1 has none): C = alpha * (A B) + beta * C, formed in
 * fp32 from the accumulators (after the W-combination of Eq. 6) and rounded once.  C is read only when beta != 0,
 * so it may then not hold NaN or Inf where a finite result is wanted; with beta == 0 its old contents are
 * ignored.  b_layout 0: B given K x N as in lcma_gemm; 2: W given N x K as in lcma_gemm_nt.  alpha = 1, beta = 0
 * gives the result of those calls bit for bit.  Everything else (sizes, alignment, errors) as for lcma_gemm;
 * ARG for another b_layout or a NaN factor. */
lcma_status lcma_gemm_ex(float alpha, float beta, int b_layout, int64_t M, int64_t N, int64_t K,
                         const void *A, int64_t lda, const void *B, int64_t ldb,
                         void *C, int64_t ldc, lcma_dtype dtype,
                         const lcma_scheme *scheme, void *stream);

/* Generated kernels ("variants": one per scheme x dtype x tile shape x dataflow, Sec. 3.1
 * Automated Code Generation).  lcma_gemm picks the preferred variant that fits the shape;
 * lcma_gemm_variant runs the named one (same contract as lcma_gemm; the scheme is the one
 * the variant was generated for).  Names look like "strassen_bf16_t128x64x16_c7".
 */
int lcma_variant_count(void);
/* Name of the scheme with id `scheme_id` as used in "builtin:<name>" ("plain" for LCMA_PLAIN), or NULL.
 * Ids 1..3 are the paper's schemes (the enum above); every further scheme file that was present when
 * the library was built (Sec. 3.1: kernels are generated per scheme) has an id from 4 up to
 * lcma_scheme_id_max().  lcma_select chooses among the paper's schemes only. */
const char *lcma_scheme_name(int scheme_id);
int lcma_scheme_id_max(void);
const char *lcma_variant_name(int index); /* NULL when out of range */
/* Describes variant `index`: builtin scheme id, dtype, tile sizes and the granules m*TM, n*TN,
 * k*TK in which it works through M, N, K (any pointer may be NULL).  Sizes are padded up to the
 * granules (a tile costs the same whether it is full or mostly padding). */
lcma_status lcma_variant_info(int index, int *scheme_id, int *dtype, int *TM, int *TN, int *TK,
                              int *mult_M, int *mult_N, int *mult_K);
lcma_status lcma_gemm_variant(const char *variant, int64_t M, int64_t N, int64_t K,
                              const void *A, int64_t lda, const void *B, int64_t ldb,
                              void *C, int64_t ldc, void *stream);
/* 1 when variant `index` takes the output of lcma_prepare_b in place of B (its B argument in
 * lcma_gemm_variant is then that buffer and ldb is ignored), 0 when it takes B, -1 when out of range. */
int lcma_variant_prepared(int index);
/* What variant `index` takes as its B argument in lcma_gemm_variant: 0 the K x N matrix B, 1 the
 * output of lcma_prepare_b, 2 the N x K matrix W of lcma_gemm_nt (ldb is then its leading
 * dimension); 3: a stage kernel of lcma_gemm_unfused, which lcma_gemm_variant refuses (ARG);
 * -1 when out of range. */
int lcma_variant_b_layout(int index);

/* Offline Combine B (Eq. 4; Algorithm 2, stage 2).  The paper's end-to-end evaluation runs this stage
 * once for static weights B; lcma_gemm_prepared then multiplies any number of A against the result.
 *
 * lcma_prepare_b writes Bt_r = sum_{l,j} V[r,l,j] B_{l,j}, r = 1..R, into Bt (device memory owned by
 * the caller, lcma_prepared_b_bytes() bytes, 16-byte aligned): R planes, plane r holding Bt_r
 * transposed, N/n rows of K/k elements, k-contiguous, in the type the products are multiplied in
 * (fp16 for BF16 and F16 storage, fp32 for F32).  The terms of a sum are added in fp32 in ascending
 * (l, j) order and the sum is rounded once, to nearest-even.  B: device, K x N row-major, ldb in
 * elements (multiple of 16 bytes).  N and K must be multiples of 16 bytes of elements; the planes
 * hold N/n rows and K/k columns padded with zeros to multiples of 64 and of 32 (16 for F32); both
 * buffers stay below 2 GiB, and the padded N/n is at most 65535 * 64 (lcma_prepare_bt: 65535 * 16), else SHAPE.
 * Asynchronous on `stream`.  Errors: ARG, BRENT, SHAPE, DTYPE, NOKERNEL
 * (no prepared-B kernels were generated for this scheme and dtype), HIP.
 *
 * lcma_prepared_b_bytes returns R * (padded N/n) * (padded K/k) * element size, or -1 for a bad
 * argument.
 *
 * lcma_gemm_prepared computes what lcma_gemm computes, C = A B, with Bt in place of B: Combine A
 * (Eq. 3) on MFMA fragments, H_r (Eq. 5) and the W-combination (Eq. 6) in fp32, nothing written to
 * device memory but C.  Same contract for A, C, sizes, alignment and errors as lcma_gemm; `scheme`
 * must be the one Bt was prepared with (not checked) and is required.
 */
int64_t lcma_prepared_b_bytes(const lcma_scheme *scheme, int64_t N, int64_t K, lcma_dtype dtype);
lcma_status lcma_prepare_b(int64_t N, int64_t K, const void *B, int64_t ldb, lcma_dtype dtype,
                           const lcma_scheme *scheme, void *Bt, void *stream);
/* lcma_prepare_b for weights stored N x K row-major (W[n][k] = B[k][n], the layout of a linear
 * layer's weight; ldw in elements): same output, bit for bit, same contract and errors. */
lcma_status lcma_prepare_bt(int64_t N, int64_t K, const void *W, int64_t ldw, lcma_dtype dtype,
                            const lcma_scheme *scheme, void *Bt, void *stream);
lcma_status lcma_gemm_prepared(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                               const void *Bt, void *C, int64_t ldc, lcma_dtype dtype,
                               const lcma_scheme *scheme, void *stream);


/* ------------------------------------------------------------------ the unfused dataflows (Algorithm 1; Algorithm 2 as printed)
 * Provided to be measured against lcma_gemm (the step-wise ablation of Sec. 4.5); for 16-bit storage at large shapes level 1
 * is the faster form on MI355X, and lcma_gemm_ws (below) chooses between the two.
 *
 * lcma_gemm_unfused computes C = A B like lcma_gemm, with intermediate results in device memory:
 *   level 1  Algorithm 1: four stages, each through device memory: Combine A (Eq. 3) writes At_r,
 *            Combine B (Eq. 4) writes Bt_r, one batched launch of the plain MFMA GEMM writes
 *            H_r = At_r Bt_r (Eq. 5), Combine H (Eq. 6) reads the H_r and writes C;
 *   level 2  Algorithm 2 as the paper runs it: Combine A and Combine B as above, then one kernel that
 *            multiplies group by group and applies W to the fp32 accumulators (H_r stays on chip).
 * At_r and Bt_r are stored in the type the products are multiplied in (fp16 for BF16 and F16
 * storage, fp32 for F32): each is an fp32 sum (ascending block order) rounded once, to nearest-even.  H_r at level 1 is
 * the fp32 MFMA accumulation, stored in fp16 (rounded once) for BF16 and as it is, in fp32, for F16 and F32: fp16 planes
 * carry no more bits than an fp16 C, and their roundings would put the result past four times the plain kernel's error.
 * <3,3,3;23> with F16 storage at level 1 works on 25 planes instead of 23: products 4 and 7 (three blocks on either side)
 * have the remainder of rounding their left combination to fp16 stored as a further plane and multiplied with a second
 * copy of Bt_r, both products entering Eq. 6 with the W row of r (without it the result lies at 4.04 times the plain
 * kernel's error, with it at 3.8, where the fused kernels of the scheme are for the same reason).
 * C is rounded once from fp32.
 * A, B, C, sizes, alignment, padding and errors as for lcma_gemm; `scheme` is required and must be
 * one of the paper's (NOKERNEL otherwise).  workspace: device memory, 256-byte aligned, at least
 * lcma_unfused_workspace_bytes() bytes (-1 for bad arguments), owned by the caller, overwritten.  Every set of planes stays
 * below 2 GiB and the padded M/m is at most 65535 * 16 (SHAPE otherwise).
 * reuse_bt != 0 skips Combine B: the Bt_r left in the workspace by an earlier call with the same B, scheme,
 * dtype, N and K are used (the paper's offline Combine B for static weights).  The Bt_r planes lie at the start
 * of the workspace and depend on N and K alone, so M may differ between such calls.
 * Asynchronous on `stream`; nothing is launched when an argument is rejected.
 */
int64_t lcma_unfused_workspace_bytes(int64_t M, int64_t N, int64_t K, lcma_dtype dtype,
                                     const lcma_scheme *scheme);
/* Split-Group Parallelism (Sec. 3.2) in the batched GEMM of level 1 (16-bit storage) and of lcma_gemm_nt_ws: the steps of all
 * tile-products are numbered tile-product-major and handed to persistent work-groups in contiguous ranges of
 * ceil(total / work-groups), so a tile-product may straddle work-groups; a work-group that holds only a piece writes fp32
 * partial sums to scratch and a second kernel adds the pieces in ascending work-group order (no atomics) and rounds once.
 * It is used when the time model prefers it to one tile-product per work-group (a poorly filled last round) AND the
 * workspace holds lcma_split_group_scratch_bytes() bytes beyond lcma_unfused_workspace_bytes(); results on float inputs
 * then differ from the other schedule in the last bit (the partial sums are cut elsewhere). */
int64_t lcma_split_group_scratch_bytes(void);
/* Plain GEMM C = A x W^T for weights stored N x K (as lcma_gemm_nt with scheme == NULL; BF16 and F16) on the kernel of the
 * batched stage, with a workspace (device, 256-byte aligned, lcma_split_group_scratch_bytes() bytes, overwritten; NULL or
 * fewer bytes: never split) that lets it hand the steps of all tiles out in Split-Group ranges: the split-K form of a plain
 * GEMM, chosen when the tiles alone would leave much of the chip idle (few tiles, long K).  K not a multiple of 64 and F32
 * are passed on to lcma_gemm_nt.  Integer-valued inputs give lcma_gemm_nt's bits; float inputs agree to the last bit or two
 * (the fp32 sums are cut differently).  Everything else as for lcma_gemm_nt. */
lcma_status lcma_gemm_nt_ws(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *W, int64_t ldw,
                            void *C, int64_t ldc, lcma_dtype dtype, void *workspace, int64_t workspace_bytes, void *stream);
lcma_status lcma_gemm_unfused(int level, int64_t M, int64_t N, int64_t K,
                              const void *A, int64_t lda, const void *B, int64_t ldb,
                              void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                              void *workspace, int64_t workspace_bytes, int reuse_bt, void *stream);

/* lcma_gemm / lcma_gemm_nt with a workspace (Sec. 3.3, the Decision Module applied to the dataflows of one scheme): the same
 * product C = A x B (b_layout 0: B given K x N as in lcma_gemm) or C = A x W^T (b_layout 2: W given N x K as in lcma_gemm_nt),
 * run as the fused kernel of those calls or as Algorithm 1 (lcma_gemm_unfused level 1; for N x K weights its Combine B reads
 * W without transposing), whichever the time model (lcma_predict_seconds against lcma_predict_unfused_seconds with Combine
 * B counted) predicts faster for the shape.
 * workspace: device memory, 256-byte aligned, overwritten; Algorithm 1 is considered only when it holds at least
 * lcma_unfused_workspace_bytes() bytes (lcma_split_group_scratch_bytes() more let its GEMM stage split tile-products
 * between work-groups); NULL, too small, a scheme that is not built in, a shape that Algorithm 1 does not take, or F16
 * storage with a scheme that sums more than 4 blocks in a row of U or V and whose stage kernels do not compensate for it
 * (its fp16 combinations would put Algorithm 1 past four times the plain kernel's error; the kernels of <3,3,3;23> do
 * compensate, see lcma_gemm_unfused): the fused kernel.  scheme == NULL: the plain product
 * (b_layout 2: lcma_gemm_nt_ws, which uses the workspace for its Split-Group schedule).
 * *dataflow (may be NULL) receives what ran: 0 = the fused kernel or the plain product, 1 = Algorithm 1.  The two dataflows
 * round differently (Algorithm 1 stores the products H_r: in fp16 for BF16, in fp32 for F16 and F32): each meets the error
 * bounds stated for it, their results are not bit-identical.  Errors: ARG for another b_layout, else those of the call
 * that ran. */
lcma_status lcma_gemm_ws(int b_layout, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                         void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                         void *workspace, int64_t workspace_bytes, int *dataflow, void *stream);

/* lcma_gemm_unfused for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the planes live in a 32 MiB buffer that is part of
 * the library's device image (lcma_static_scratch_bytes() bytes, one copy per GPU, held until the process ends).
 * The call allocates nothing and calls no allocating routine.  Shapes whose planes need more than the buffer
 * (lcma_unfused_workspace_bytes() > lcma_static_scratch_bytes(), e.g. Strassen bf16 beyond about 1700^3) are
 * rejected with LCMA_ERR_SHAPE and nothing is launched.  Every call on a GPU uses that GPU's one buffer: calls on
 * different streams of one GPU that overlap in time race; calls on one stream are ordered.  reuse_bt refers to the
 * Bt_r planes left by the previous call on the same GPU.  Everything else as for lcma_gemm_unfused. */
int64_t lcma_static_scratch_bytes(void);
lcma_status lcma_gemm_unfused_static(int level, int64_t M, int64_t N, int64_t K,
                                     const void *A, int64_t lda, const void *B, int64_t ldb,
                                     void *C, int64_t ldc, lcma_dtype dtype, const lcma_scheme *scheme,
                                     int reuse_bt, void *stream);

/* The Decision Module (Sec. 3.3) over both dataflows this library runs: predicted seconds of Algorithm 1
 * (lcma_gemm_unfused level 1) for a built-in scheme id, stage by stage (Combine A, Combine B unless
 * combine_b_offline, the batched GEMM, Combine H; negative when the scheme has no stage kernels), and the
 * choice with the smallest predicted time among plain, the fused kernels and Algorithm 1 of the paper's
 * schemes.  dataflow: 0 = lcma_gemm (fused; scheme_id LCMA_PLAIN means the plain GEMM), 1 = lcma_gemm_unfused
 * level 1.  Pure host arithmetic. */
typedef struct { int scheme_id; int dataflow; double seconds; } lcma_choice;
double lcma_predict_unfused_seconds(int scheme_id, int64_t M, int64_t N, int64_t K, lcma_dtype dtype,
                                    int combine_b_offline);
lcma_status lcma_select_dataflow(int64_t M, int64_t N, int64_t K, lcma_dtype dtype,
                                 int combine_b_offline, lcma_choice *out);

/* ------------------------------------------------------------------ FP8 (Sec. 4.1 experimental setup; Sec. 4.3 fused quantisation)
 * The paper's FP8 workflow: bf16 operands, quantised to FP8 E4M3 with one scale per 1 x 128 block along K, multiplied
 * block-scaled; in the LCMA form the quantisation is fused into the Combine A stage.  As built here:
 *   - E4M3 is the OCP format (bias 7, largest finite value 448, no infinities); conversion rounds to nearest, ties to even;
 *   - a scale is a power of two 2^e stored as the byte e + 127 (E8M0), e the smallest integer with amax <= 448 * 2^e over the
 *     128 values of the block (e = 0 for an all-zero block): dividing by it is exact, and MI355X's scaled matrix
 *     instruction applies it in hardware;
 *   - both operands are scaled along K: A per row, the weights per row of the N x K matrix W (C = A x W^T);
 *   - the sums of Eq. 3 / Eq. 4 are formed in fp32 in ascending block order before they are quantised; products
 *     accumulate in fp32; C is bf16, rounded once.
 * Code matrices hold one byte per element, rows of lcma_fp8_code_pitch(K) = K rounded up to 128 bytes (the padding holds
 * zero codes); scale matrices hold lcma_fp8_scale_pitch(K) bytes per row (K/128 rounded up, then up to a multiple of 4).
 * All pointers are device pointers owned by the caller; calls are asynchronous on `stream`; K must be a multiple of 8;
 * every matrix stays below 2 GiB.  Errors: ARG, SHAPE, BRENT, NOKERNEL, HIP; nothing is launched on error.
 *
 * lcma_fp8_quantize   X: rows x K bf16 (ldx in elements, 16-byte aligned) -> Q: rows x code pitch, S: rows x scale pitch.
 * lcma_fp8_gemm_nt    plain block-scaled product: C[M x N] (bf16, 16-byte aligned, ldc in elements and a multiple of 8, N a
 *                     multiple of 8) from the codes and scales of A (M x K) and of W (N x K), each as written by
 *                     lcma_fp8_quantize.
 * lcma_fp8_prepare_w  offline Combine B (Eq. 4) for static weights W (N x K bf16) with the quantisation fused in: writes R
 *                     planes of codes and their scales into Wp (lcma_fp8_prepared_w_bytes() bytes, 256-byte aligned).
 * lcma_fp8_gemm_lcma  C = A x W^T by Algorithm 1 on FP8 operands: Combine A (Eq. 3) from the bf16 matrix A with the
 *                     quantisation fused in, one batched launch of the block-scaled GEMM over the R planes (Eq. 5, products
 *                     stored in fp16), Combine H (Eq. 6, fp32 sums in ascending r, one rounding to bf16).  workspace:
 *                     lcma_fp8_workspace_bytes() bytes, 256-byte aligned, overwritten.  N must be a multiple of 8 as well.
 * The byte counts return -1 for a bad argument. */
int64_t lcma_fp8_code_pitch(int64_t K);
int64_t lcma_fp8_scale_pitch(int64_t K);
lcma_status lcma_fp8_quantize(int64_t rows, int64_t K, const void *X, int64_t ldx, void *Q, void *S, void *stream);
lcma_status lcma_fp8_gemm_nt(int64_t M, int64_t N, int64_t K, const void *Aq, const void *Sa,
                             const void *Wq, const void *Sw, void *C, int64_t ldc, void *stream);
int64_t lcma_fp8_prepared_w_bytes(const lcma_scheme *scheme, int64_t N, int64_t K);
lcma_status lcma_fp8_prepare_w(int64_t N, int64_t K, const void *W, int64_t ldw, const lcma_scheme *scheme,
                               void *Wp, void *stream);
int64_t lcma_fp8_workspace_bytes(const lcma_scheme *scheme, int64_t M, int64_t N, int64_t K);
lcma_status lcma_fp8_gemm_lcma(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *Wp,
                               void *C, int64_t ldc, const lcma_scheme *scheme,
                               void *workspace, int64_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------ Decision Module (Sec. 3.3)
 * lcma_select: predicted-fastest algorithm for the shape on MI355X among
 * {plain, <2,2,2;7>, <4,4,4;49>, <3,3,3;23>}; returns a built-in scheme id, or a
 * negative value on bad arguments.  Pure host arithmetic.
 */
int lcma_select(int64_t M, int64_t N, int64_t K, lcma_dtype dtype);

/* The hardware tuple of Sec. 3.3: multiply rate, add rate (operations/s) and off-chip
 * bandwidth in ELEMENTS/s of the dtype. */
typedef struct { double flops_mul, flops_add, beta; } lcma_hw;
/* Published MI355X figures for a dtype (dense MFMA peak, fp32 vector rate, 8 TB/s). */
lcma_status lcma_hw_mi355x(lcma_dtype dtype, lcma_hw *out);

/* Per-stage operation and element-traffic counts of Table 2, and the stage times of the
 * roofline rule of Sec. 3.3 (time = max(flops/rate, elements/beta)). Index: 0 Combine A,
 * 1 Combine B, 2 GEMM, 3 Combine H.  scheme == NULL gives the standard GEMM in slot 2. */
typedef struct { double flops[4], elems[4], seconds[4]; } lcma_stage_costs;
lcma_status lcma_model_stages(const lcma_scheme *s, int64_t M, int64_t N, int64_t K,
                              const lcma_hw *hw, lcma_stage_costs *out);
/* Left-hand sides of Eq. 8 (plain GEMM intensity), Eq. 9 and Eq. 10 (fused Combine H),
 * to be compared with flops_mul / beta. */
lcma_status lcma_model_intensity(const lcma_scheme *s, int64_t M, int64_t N, int64_t K,
                                 double *eq8, double *eq9, double *eq10);
/* The model lcma_select uses for THIS library's fused kernels: predicted seconds of the
 * preferred variant of built-in `scheme_id` (LCMA_PLAIN..LCMA_LADERMAN) on MI355X, or a
 * negative value when no variant fits the shape. */
double lcma_predict_seconds(int scheme_id, int64_t M, int64_t N, int64_t K, lcma_dtype dtype);

/* ------------------------------------------------------------------ measurement aids
 * Process-wide settings; none but the last changes a result.  lcma_set_tuning(key, value) sets one (value "" or NULL restores the
 * default); the initial values come from the environment variables named below, which are read ONCE, at the first
 * call that needs them.  Errors: ARG for an unknown key.
 *   "variant"          LCMA_VARIANT=<name>          lcma_gemm / lcma_gemm_prepared run this generated kernel when it belongs
 *                                                   to the requested scheme, dtype and layout (otherwise ignored)
 *   "unfused_variant"  LCMA_UNFUSED_VARIANT=<name>  the same for the GEMM stage of lcma_gemm_unfused
 *   "panel"            LCMA_PANEL=<n>               width, in tiles, of the column panels of the tile order (default 8; the
 *                                                   plane GEMM then takes 7, 6 or 5 where that divides the columns of tiles
 *                                                   and 8 does not)
 *   "batch_order"      LCMA_BATCH_ORDER=1           batched GEMM of lcma_gemm_unfused level 1 in group-major instead of
 *                                                   product-major order
 *   "schedule"         LCMA_SCHEDULE=static|split|persist   batched GEMM stages: one tile-product per work-group, contiguous
 *                                                   ranges of steps per persistent work-group (Sec. 3.2, Split-Group
 *                                                   Parallelism), or persistent work-groups that take whole tile-products in
 *                                                   turn; default: whichever the time model prefers
 *   "unfused_stages"   LCMA_UNFUSED_STAGES=<mask>   for timing one stage of lcma_gemm_unfused alone: bit 0 Combine A, bit 1
 *                                                   Combine B, bit 2 the GEMM stage, bit 3 Combine H (default 15, all).  The one
 *                                                   setting that is not result-neutral: a stage switched off leaves its output
 *                                                   as an earlier call wrote it, so C is only valid with all four on.
 */
lcma_status lcma_set_tuning(const char *key, const char *value);

/* ------------------------------------------------------------------ tile scheduling (Sec. 3.2, Split-Group Parallelism)
 * Wave counts for `groups` groups of R tile-products on `units` compute units:
 * tile-level scheduling needs ceil(groups*R/units) waves, group-level ceil(groups/units)*R.
 */
lcma_status lcma_sched_waves(int64_t groups, int R, int units,
                             int64_t *tile_level, int64_t *group_level);
/* Split-Group assignment: tile-products are numbered group-major (job = group*R + r) and
 * unit u of `units` owns the contiguous range [*begin, *end) with capacity
 * ceil(total/units); a group can therefore straddle at most two units. */
lcma_status lcma_sched_range(int64_t groups, int R, int units, int unit,
                             int64_t *begin, int64_t *end);

const char *lcma_status_str(lcma_status st);
const char *lcma_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LCMA_H */
