// Kernel argument block shared by the host launcher and the generated gfx950 kernels.
//
// Ragged M and N.  The blocks of the scheme are cut from the matrices padded (virtually, with zeros)
// to whole tiles: the block steps below are those of the padded sizes, the byte extents are the true
// ones.  Rows past M fall outside the extents: gfx950 range-checks voffset + soffset per lane against
// the descriptor, returns 0 for such loads and drops such stores (measured).  Columns past N would
// alias the next row, so lanes that own them get an offset at the end of the extent instead.
// Ragged K: rows of B past K fall outside the extent as well; columns of A past K (only in the last
// block column, only in its last y steps) get the offset at the end of the extent, decided in those
// steps alone.
#pragma once
#include <stdint.h>

namespace lcma {

struct Params {
    const void *A;
    const void *B;                      // prepared-B kernels: the R planes written by the Combine-B kernel
    void *C;
    uint32_t a_bytes, b_bytes, c_bytes; // byte extents of the three matrices (< 2 GiB each)
    uint32_t lda_b, ldb_b, ldc_b;       // leading dimensions in BYTES
    uint32_t a_brow, a_bcol;            // byte step from block A_{i,l} to A_{i+1,l} / A_{i,l+1}
    uint32_t b_brow, b_bcol;            // byte step from block B_{l,j} to B_{l+1,j} / B_{l,j+1}
                                        // (prepared B: ldb_b = row pitch of a plane, b_brow = plane stride)
    uint32_t c_brow, c_bcol;            // byte step from block C_{i,j} to C_{i+1,j} / C_{i,j+1}
    int32_t nx, nz, ny;                 // tiles per block along M/m, N/n and K/k (Algorithm 2's x, z, y ranges in tiles)
    int32_t panel;                      // width (in z tiles) of a column panel in the tile order
    uint32_t n_row_b;                   // N * element size: columns at or beyond it are padding (read as 0, never written)
    uint32_t k_row_b;                   // K * element size: columns of A at or beyond it are padding (read as 0)
    uint32_t k_tail_b;                  // byte column inside a block from which the LAST block column of A may
                                        // run past K: K*ES - (k-1)*a_bcol, rounded down to whole tiles
    int32_t batch_order = 0;            // batched kernels: 0 = product-major (all tiles of product r, then r + 1: concurrent
                                        // work-groups share r, the paper's Cache-Aware order), 1 = group-major (the R products
                                        // of a tile position next to each other), kept to measure the difference
    float alpha = 1.f, beta = 0.f;      // C = alpha * (A B) + beta * C, in fp32 before the one rounding; C is read only when beta != 0
};

// Argument block of the offline Combine-B kernels.
struct PrepParams {
    const void *B;
    void *Bt;
    uint32_t b_bytes, bt_bytes; // byte extents (< 2 GiB each)
    uint32_t ldb_b;             // leading dimension of B in bytes
    uint32_t b_brow, b_bcol;    // byte step from block B_{l,j} to B_{l+1,j} / B_{l,j+1}
    uint32_t bt_ld_b;           // row pitch of a plane in bytes = (K/k) * ES
    uint32_t bt_plane_b;        // plane stride in bytes = (N/n) * (K/k) * ES
    int32_t bk, bn;             // K/k, padded N/n
    uint32_t n_row_b;           // N * element size of B: columns at or beyond it are read as 0
};

// Argument block of the stand-alone Combine-H kernels (stage 4 of Algorithm 1).
struct CombHParams {
    const void *H;
    void *C;
    uint32_t h_bytes, c_bytes; // byte extents (< 2 GiB each)
    uint32_t h_ld_b;           // row pitch of a plane in bytes
    uint32_t h_plane_b;        // plane stride in bytes
    uint32_t ldc_b;            // leading dimension of C in bytes
    uint32_t c_brow, c_bcol;   // byte step from block C_{i,j} to C_{i+1,j} / C_{i,j+1}
    uint32_t n_row_b;          // N * element size: columns at or beyond it are never written
};

// Argument blocks of the FP8 kernels (E4M3 codes, one E8M0 scale byte per 1 x 128 block along K).
// Argument block of the plane GEMM (csrc/lcma_plane_gemm.hpp): k-contiguous operands, FP8 codes with scale bytes or
// 16-bit elements, plain or batched over planes, handed out in contiguous ranges of steps (Sec. 3.2, Split-Group).
struct PlaneGemmParams {
    const void *A, *SA, *B, *SB;                            // SA, SB: scale bytes (FP8 only)
    void *C;
    uint32_t a_bytes, sa_bytes, b_bytes, sb_bytes, c_bytes; // byte extents (< 2 GiB each; all planes of a batch)
    uint32_t lda_b, ldb_b;                                  // row pitch of the operands in bytes
    uint32_t lsa_b, lsb_b;                                  // row pitch of the scale matrices in bytes (multiples of 4)
    uint32_t ldc_b;                                         // row pitch of C in bytes
    uint32_t a_plane, sa_plane, b_plane, sb_plane, c_plane; // batched: byte step from plane r to r + 1
    int32_t nx, nz, ny;                                     // tiles along M and N; steps of 128 bytes along K
    int32_t panel;                                          // width (in z tiles) of a column panel of the tile order
    uint32_t n_row_b;                                       // N * 2: columns of C at or beyond it are never written
    int32_t jobs;                                           // tile-products: planes * nx * nz
    int32_t units;                                          // persistent work-groups launched
    int32_t interleave;                                     // persistent kernel: 0 = work-group u owns the steps [u * cap, (u + 1) * cap);
                                                            // whole tile-products in turn: 1 = u, u + units, ... (rounds of consecutive
                                                            // ones), 2 = each XCD an eighth of them (units is a multiple of 8)
    int64_t cap;                                            // steps per work-group: ceil(jobs * ny / units)
    void *partial;                                          // fp32 scratch for pieces: 2 slots of TM * TN floats per work-group
                                                            // (never touched when cap is a multiple of ny)
};

struct Fp8QuantParams {
    const void *X;             // bf16 source, row-major
    void *Q, *S;               // codes and scale bytes (first plane)
    uint32_t x_bytes, q_bytes, s_bytes;
    uint32_t ldx_b;            // row pitch of X in bytes
    uint32_t x_brow, x_bcol;   // combine kernels: byte step from block (j, l) of X to (j + 1, l) / (j, l + 1)
    uint32_t ldq_b, lds_b;     // row pitch of a plane of codes / of scale bytes
    uint32_t q_plane, s_plane; // byte step between planes
    uint32_t k_row_b;          // K * 2: columns of X at or beyond it read as zero
    int32_t rows;              // rows of a plane (padded); rows past the extent of X read as zero
};

} // namespace lcma
