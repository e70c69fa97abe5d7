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
// each block that any product uses (two 16-byte vectors per thread and block, kept in registers as
// loaded), and for each r forms the sums, transposes them through LDS and writes 64 rows of KT
// k-contiguous elements: 128 bytes, a whole line.  HBM traffic is the compulsory K*N*ES in +
// R/(k*n) * K*N*ES out.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

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

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>) in turn.  The loops over the products of a scheme are
// written with this instead of `#pragma unroll`: every pass selects its sum by a switch over the product, which folds
// only for a constant, and the unroller gives up on 49 passes of a body that still holds 49 cases (the loop then
// stays, with a branch tree per element).
template <class F, int... Is> LCMA_DEV void for_each_const(F &&f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F> LCMA_DEV void for_each_const(F &&f) { for_each_const(f, std::make_integer_sequence<int, N>{}); }

// Element e of a raw 16-byte vector as fp32 (exact).
template <class IN> struct Elem;
template <> struct Elem<F32> {
    static LCMA_DEV float get(u32x4 raw, int e) {
        const uint32_t w = raw[e]; // (a copy: __builtin_bit_cast applied to the vector element itself reads element 0)
        return __builtin_bit_cast(float, w);
    }
};
template <> struct Elem<BF16> {
    static LCMA_DEV float get(u32x4 raw, int e) {
        return __builtin_bit_cast(float, (e & 1) ? raw[e >> 1] & 0xffff0000u : raw[e >> 1] << 16);
    }
};
template <> struct Elem<F16> {
    static LCMA_DEV float get(u32x4 raw, int e) { return (float)__builtin_bit_cast(f16x8, raw)[e]; }
};

// The blocks stay in registers as loaded and are widened where a sum uses them.  Before every product the compiler is
// made to forget what it derived from them: the sums of different products share parts, and kept alive across the R
// products of a scheme with many blocks (16 for <4,4,4;49>) those parts fill the register file to one wave per SIMD,
// which for a kernel that only waits for memory is three times slower.
template <int NB> LCMA_DEV void forget_derived(u32x4 (&raw)[NB]) {
#pragma unroll
    for (int t = 0; t < NB; ++t) asm volatile("" : "+v"(raw[t]));
}

// 64-byte segments of an output row that one work-group of the K x N kernel writes: two, i.e. whole 128-byte lines (with
// one: 9 % slower for <2,2,2;7>, 26 % for <4,4,4;49>).  A launcher is handed the number of segments in K/k and divides it
// by this.
constexpr int kPrepBSegments = 2;

// CH (generated): NB raw blocks with b_l(t), b_j(t); NP outputs; comb(in, r) = Eq. 4 for product r on floats;
// residual(r): plane r holds what rounding that sum to fp16 loses instead of the rounded sum (16-bit types only).
template <class IN, class CT, class CH> LCMA_DEV void prepare_b_tile(const PrepParams &p) {
    constexpr int ES = IN::ES, EPT = 16 / ES;       // elements per 16-byte vector
    constexpr int KV = kPrepBSegments;
    constexpr int KS = 64 / ES;                     // k rows per 64-byte segment of an output row (32 or 16)
    constexpr int KT = KV * KS;                     // k rows of the tile
    constexpr int PITCH = KV * 64 + 16;             // LDS row pitch in bytes, 16-byte aligned
    static_assert(CT::ES == ES, "the output keeps the element size");
    __shared__ __attribute__((aligned(16))) char tile[64 * PITCH];
    const auto rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.B), 0, (int)p.b_bytes, 0x00020000);
    const auto rt = __builtin_amdgcn_make_buffer_rsrc(p.Bt, 0, (int)p.bt_bytes, 0x00020000);
    const int tid = threadIdx.x;
    // work-groups that start together cover consecutive pieces of the same 64 rows of the planes (23 % faster at
    // 8192 x 14336 x 4096 than the other order, which reads B in whole rows instead)
    const int z0 = blockIdx.y * 64, y0 = blockIdx.x * KT;
    // a lane takes KV consecutive k rows and consecutive lanes the next ones, so that the transposed LDS writes are
    // whole dwords at consecutive addresses
    const int ky = tid % KS, tx = tid / KS; // tx: which vector of EPT columns
    u32x4 in[KV][CH::NB];
#pragma unroll
    for (int v = 0; v < KV; ++v)
#pragma unroll
        for (int t = 0; t < CH::NB; ++t) {
            const int k = y0 + KV * ky + v;
            const uint32_t colb = (uint32_t)CH::b_j(t) * p.b_bcol + (uint32_t)(z0 + tx * EPT) * ES;
            // columns past N are padding, and so are rows past K/k (they belong to the next block): read from the end
            // of the extent, which returns zero
            const uint32_t off = colb < p.n_row_b && k < p.bk ? (uint32_t)CH::b_l(t) * p.b_brow + (uint32_t)k * p.ldb_b + colb
                                                              : p.b_bytes;
            in[v][t] = __builtin_amdgcn_raw_buffer_load_b128(rb, (int)off, 0, 0);
        }
    for_each_const<CH::NP>([&](auto rc_) {
        constexpr int r = decltype(rc_)::value;
#pragma unroll
        for (int v = 0; v < KV; ++v) forget_derived(in[v]);
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            float o[KV];
#pragma unroll
            for (int v = 0; v < KV; ++v) {
                float col[CH::NB];
#pragma unroll
                for (int t = 0; t < CH::NB; ++t) col[t] = Elem<IN>::get(in[v][t], e);
                o[v] = CH::comb(col, r);
                if constexpr (ES == 2) {
                    if (CH::residual(r)) o[v] -= (float)(_Float16)o[v]; // what rounding the sum loses (exact in fp32)
                }
            }
            char *dst = tile + (tx * EPT + e) * PITCH + KV * ky * ES;
            if constexpr (ES == 2) { // one rounding, nearest-even
                if constexpr (KV == 2) {
                    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
                    const f16x2 h = {(_Float16)o[0], (_Float16)o[1]};
                    *(f16x2 *)dst = h;
                } else {
                    *(_Float16 *)dst = (_Float16)o[0];
                }
            } else {
#pragma unroll
                for (int v = 0; v < KV; ++v) ((float *)dst)[v] = o[v];
            }
        }
        __syncthreads();
        // read back: 4 * KV threads per output row, 16 bytes each
#pragma unroll
        for (int i = 0; i < KV; ++i) {
            const int idx = tid + 256 * i, rn = idx / (4 * KV), rc = idx % (4 * KV);
            const u32x4 v = *(const u32x4 *)(tile + rn * PITCH + rc * 16);
            const uint32_t kb = (uint32_t)y0 * ES + rc * 16; // byte column in the row of the plane
            // a segment past K/k is dropped (stored to the end of the extent)
            const uint32_t off = kb < (uint32_t)p.bk * ES ? (uint32_t)r * p.bt_plane_b + (uint32_t)(z0 + rn) * p.bt_ld_b + kb : p.bt_bytes;
            // (16-byte store: the scalar-offset field stays a literal zero, see Ctx::store_c in lcma_device.hpp)
            __builtin_amdgcn_raw_buffer_store_b128(v, rt, (int)off, 0, 0);
        }
        __syncthreads();
    });
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
    // 256 threads: 16 rows (n) x 16 vectors (k) of every block; work-groups that start together cover consecutive
    // pieces of the same rows (whole rows of the planes are written at a time: 19 % faster at 4096^3 than row-major order)
    const int rn = blockIdx.y * 16 + (int)threadIdx.x / 16;
    const uint32_t kb = (uint32_t)(blockIdx.x * 16 + (int)threadIdx.x % 16) * 16; // byte column inside a block
    if (kb >= p.bt_ld_b) return; // past the padded K/k (whole work-group columns only when K/k < 256 B)
    u32x4 in[CH::NB];
#pragma unroll
    for (int t = 0; t < CH::NB; ++t) {
        // block B_{l,j} of B is block (j, l) of W; rows past N lie outside the extent, columns past K
        // would alias the next row
        const uint32_t colb = (uint32_t)CH::b_l(t) * p.b_bcol + kb;
        const uint32_t off = colb < p.n_row_b ? (uint32_t)CH::b_j(t) * p.b_brow + (uint32_t)rn * p.ldb_b + colb : p.b_bytes;
        in[t] = __builtin_amdgcn_raw_buffer_load_b128(rb, (int)off, 0, 0);
    }
    for_each_const<CH::NP>([&](auto rc_) {
        constexpr int r = decltype(rc_)::value;
        forget_derived(in);
        u32x4 v;
        if constexpr (ES == 2) {
            f16x8 h;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                float col[CH::NB];
#pragma unroll
                for (int t = 0; t < CH::NB; ++t) col[t] = Elem<IN>::get(in[t], e);
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
                for (int t = 0; t < CH::NB; ++t) col[t] = Elem<IN>::get(in[t], e);
                f[e] = CH::comb(col, r);
            }
            v = __builtin_bit_cast(u32x4, f);
        }
        const uint32_t off = (uint32_t)r * p.bt_plane_b + (uint32_t)rn * p.bt_ld_b + kb;
        // (16-byte store: the scalar-offset field stays a literal zero, see Ctx::store_c in lcma_device.hpp)
        __builtin_amdgcn_raw_buffer_store_b128(v, rt, (int)off, 0, 0);
    });
}

} // namespace lcma
