// Offline Combine B for gfx950 (paper Eq. 4 / Algorithm 2 stage 2, run once for static weights as in
// the paper's end-to-end evaluation): Bt_r = sum_{l,j} V[r,l,j] B_{l,j} for r = 1..R.
//
// Output layout ("prepared B"): R planes; plane r holds Bt_r TRANSPOSED, (N/n) rows of (K/k)
// elements, k-contiguous, in the type the products are multiplied in (fp16 for bf16 and fp16
// storage, fp32 for fp32 storage).  That is the layout the MFMA B operand is read in, so the GEMM
// kernel copies tiles of it to LDS without touching them.
//
// Arithmetic: the terms of a sum are widened to fp32 (exact) and added in fp32 in ascending (l, j)
// order, the sum is rounded once, to nearest-even, to the output type.  (The fused kernels add in
// packed fp16; here the work is HBM-bound and the wider sum is free.)
//
// One work-group of 256 threads handles KT x 64 elements (k x n) of every block: it reads the tile of
// each block that any product uses (one 16-byte vector per thread and block, kept in registers as
// fp32), and for each r forms the sums, transposes them through LDS and writes 64 rows of KT
// k-contiguous elements.  HBM traffic is the compulsory K*N*ES in + R/(k*n) * K*N*ES out.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_device.hpp"

namespace lcma {

template <class IN> struct Widen;
template <> struct Widen<F32> {
    static LCMA_DEV void run(u32x4 raw, float (&out)[4]) {
        const f32x4 f = __builtin_bit_cast(f32x4, raw);
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = f[e];
    }
};
template <> struct Widen<BF16> {
    static LCMA_DEV void run(u32x4 raw, float (&out)[8]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[2 * e] = __builtin_bit_cast(float, raw[e] << 16);
            out[2 * e + 1] = __builtin_bit_cast(float, raw[e] & 0xffff0000u);
        }
    }
};
template <> struct Widen<F16> {
    static LCMA_DEV void run(u32x4 raw, float (&out)[8]) {
        const f16x8 h = __builtin_bit_cast(f16x8, raw);
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (float)h[e];
    }
};

// CH (generated): NB raw blocks with b_l(t), b_j(t); NP outputs; comb(in, r) = Eq. 4 for product r on floats;
// residual(r): plane r holds what rounding that sum to fp16 loses instead of the rounded sum (16-bit types only).
template <class IN, class CT, class CH> LCMA_DEV void prepare_b_tile(const PrepParams &p) {
    constexpr int ES = IN::ES, EPT = 16 / ES;       // elements per 16-byte vector
    constexpr int KT = 64 / ES;                     // k rows of the tile (32 or 16): 64-byte output rows
    constexpr int PITCH = 80;                       // LDS row pitch in bytes (64 of data), 16-byte aligned
    static_assert(CT::ES == ES, "the output keeps the element size");
    __shared__ __attribute__((aligned(16))) char tile[64 * PITCH];
    const auto rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.B), 0, (int)p.b_bytes, 0x00020000);
    const auto rt = __builtin_amdgcn_make_buffer_rsrc(p.Bt, 0, (int)p.bt_bytes, 0x00020000);
    const int tid = threadIdx.x;
    const int z0 = blockIdx.x * 64, y0 = blockIdx.y * KT;
    // consecutive lanes take consecutive k rows, so that the transposed LDS writes fall into
    // consecutive addresses
    const int ky = tid % KT, tx = tid / KT; // tx: which vector of EPT columns
    float in[CH::NB][EPT];
#pragma unroll
    for (int t = 0; t < CH::NB; ++t) {
        const uint32_t colb = (uint32_t)CH::b_j(t) * p.b_bcol + (uint32_t)(z0 + tx * EPT) * ES;
        // columns past N are padding: read from the end of the extent, which returns zero
        const uint32_t off = colb < p.n_row_b ? (uint32_t)CH::b_l(t) * p.b_brow + (uint32_t)(y0 + ky) * p.ldb_b + colb
                                              : p.b_bytes;
        Widen<IN>::run(__builtin_amdgcn_raw_buffer_load_b128(rb, (int)off, 0, 0), in[t]);
    }
    // read-back assignment: 4 threads per output row, 16 bytes each
    const int rn = tid / 4, rc = tid % 4;
#pragma unroll
    for (int r = 0; r < CH::NP; ++r) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            float col[CH::NB];
#pragma unroll
            for (int t = 0; t < CH::NB; ++t) col[t] = in[t][e];
            float o = CH::comb(col, r);
            if constexpr (ES == 2) {
                if (CH::residual(r)) o -= (float)(_Float16)o; // what rounding the sum loses (exact in fp32)
            }
            char *dst = tile + (tx * EPT + e) * PITCH + ky * ES;
            if constexpr (ES == 2) *(_Float16 *)dst = (_Float16)o; // one rounding, nearest-even
            else *(float *)dst = o;
        }
        __syncthreads();
        const u32x4 v = *(const u32x4 *)(tile + rn * PITCH + rc * 16);
        const uint32_t off = (uint32_t)r * p.bt_plane_b + (uint32_t)(z0 + rn) * p.bt_ld_b + (uint32_t)y0 * ES + rc * 16;
        // (16-byte store: the scalar-offset field stays a literal zero, see Ctx::store_c in lcma_device.hpp)
        __builtin_amdgcn_raw_buffer_store_b128(v, rt, (int)off, 0, 0);
        __syncthreads();
    }
}

// The same stage for a weight matrix stored as N x K (row n holds the K inputs of output n, the layout
// of a linear layer's weight): W[n][k] = B[k][n].  The rows are k-contiguous already, so there is nothing
// to transpose: a thread reads one 16-byte vector per block, forms the sums and writes one 16-byte
// vector per plane.  Here PrepParams describes W: ldb_b is its row pitch, b_brow the byte step between
// block rows of W (n direction, (N/n) * ldb_b) and b_bcol between its block columns (k direction).
template <class IN, class CT, class CH> LCMA_DEV void prepare_bt_tile(const PrepParams &p) {
    constexpr int ES = IN::ES, EPT = 16 / ES;
    static_assert(CT::ES == ES, "the output keeps the element size");
    const auto rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.B), 0, (int)p.b_bytes, 0x00020000);
    const auto rt = __builtin_amdgcn_make_buffer_rsrc(p.Bt, 0, (int)p.bt_bytes, 0x00020000);
    // 256 threads: 16 rows (n) x 16 vectors (k) of every block
    const int rn = blockIdx.x * 16 + (int)threadIdx.x / 16;
    const uint32_t kb = (uint32_t)(blockIdx.y * 16 + (int)threadIdx.x % 16) * 16; // byte column inside a block
    if (kb >= p.bt_ld_b) return; // past the padded K/k (whole work-group columns only when K/k < 256 B)
    float in[CH::NB][EPT];
#pragma unroll
    for (int t = 0; t < CH::NB; ++t) {
        // block B_{l,j} of B is block (j, l) of W; rows past N lie outside the extent, columns past K
        // would alias the next row
        const uint32_t colb = (uint32_t)CH::b_l(t) * p.b_bcol + kb;
        const uint32_t off = colb < p.n_row_b ? (uint32_t)CH::b_j(t) * p.b_brow + (uint32_t)rn * p.ldb_b + colb : p.b_bytes;
        Widen<IN>::run(__builtin_amdgcn_raw_buffer_load_b128(rb, (int)off, 0, 0), in[t]);
    }
#pragma unroll
    for (int r = 0; r < CH::NP; ++r) {
        u32x4 v;
        if constexpr (ES == 2) {
            f16x8 h;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                float col[CH::NB];
#pragma unroll
                for (int t = 0; t < CH::NB; ++t) col[t] = in[t][e];
                float o = CH::comb(col, r);
                if (CH::residual(r)) o -= (float)(_Float16)o; // what rounding the sum loses (exact in fp32)
                h[e] = (_Float16)o; // one rounding, nearest-even
            }
            v = __builtin_bit_cast(u32x4, h);
        } else {
            f32x4 f;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                float col[CH::NB];
#pragma unroll
                for (int t = 0; t < CH::NB; ++t) col[t] = in[t][e];
                f[e] = CH::comb(col, r);
            }
            v = __builtin_bit_cast(u32x4, f);
        }
        const uint32_t off = (uint32_t)r * p.bt_plane_b + (uint32_t)rn * p.bt_ld_b + kb;
        // (16-byte store: the scalar-offset field stays a literal zero, see Ctx::store_c in lcma_device.hpp)
        __builtin_amdgcn_raw_buffer_store_b128(v, rt, (int)off, 0, 0);
    }
}

} // namespace lcma
