// FP8 path for gfx950 (CDNA4): E4M3 operands with one power-of-two scale per 1 x 128 block along K.
//
// The paper's FP8 workflow (Sec. 4.1, experimental setup: bf16 operands quantised to FP8 E4M3 with 1 x 128 block-wise
// scaling; Sec. 4.3: the quantisation fused into the Combine A stage) on MI355X's own terms: a scale is 2^e stored as
// the byte e + 127 (the E8M0 scale type), which the scaled matrix instruction v_mfma_scale_f32_32x32x64_f8f6f4 applies
// in hardware, so the block-scaled product costs no vector instruction per element and accumulates across the K/128
// blocks in one set of fp32 registers.  e is the smallest integer with amax <= 448 * 2^e (0 for an all-zero block):
// dividing by 2^e is exact, the one rounding is the conversion to E4M3 (nearest, ties to even).
//
// Kernels:
//   quantize_rows        bf16 matrix -> codes + scale bytes (the plain workflow, and static weights);
//   combine_quantize     Combine A (Eq. 3) or Combine B for N x K weights (Eq. 4) with the quantisation fused in: the
//                        signed sums are formed in fp32 in ascending block order (generated code) and leave the kernel
//                        as E4M3 planes with their scales;
//   the block-scaled GEMM on codes and scales (Eq. 5 on the dequantised operands) is the plane GEMM of
//   csrc/lcma_plane_gemm.hpp with FP8 operands.
// Layouts: code matrices are row-major and k-contiguous (A: M x K, W: N x K), one byte per element; a scale matrix
// has one row per row of codes and K/128 bytes per row, the row pitch padded to a multiple of 4 bytes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_prepare_b.hpp" // Elem, forget_derived, for_each_const

namespace lcma {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Smallest e with amax <= 448 * 2^e as the byte e + 127; amax = f * 2^q with f in [1, 2): 448 = 1.75 * 2^8, so
// e = q - 8 when f <= 1.75 and q - 7 otherwise.  Decided on the bits of the fp32 value, no rounding involved.
LCMA_DEV int scale_byte_of(float amax) {
    const uint32_t bits = __builtin_bit_cast(uint32_t, amax);
    if (bits == 0) return 127;
    int q = (int)(bits >> 23) - 127;
    uint32_t man = bits & 0x7fffffu;
    if ((bits >> 23) == 0) { // subnormal fp32: normalise
        const int lz = __builtin_clz(man) - 8;
        q = -126 - lz;
        man = (man << lz) & 0x7fffffu;
    }
    int e = q - 8 + (man > 0x600000u ? 1 : 0); // mantissa of 1.75 is 0x600000
    e = e < -127 ? -127 : (e > 127 ? 127 : e);
    return e + 127;
}

// Eight fp32 values scaled by 2^-e (exact) and converted to E4M3 codes, packed in two dwords.
LCMA_DEV u32x2 quantize8(const float (&v)[8], int e) {
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_ldexpf(v[0], -e), __builtin_ldexpf(v[1], -e), lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_ldexpf(v[2], -e), __builtin_ldexpf(v[3], -e), lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_ldexpf(v[4], -e), __builtin_ldexpf(v[5], -e), hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_ldexpf(v[6], -e), __builtin_ldexpf(v[7], -e), hi, true);
    return u32x2{(uint32_t)lo, (uint32_t)hi};
}

// Largest magnitude over the 16 lanes that hold one 128-element block (lanes 16g .. 16g + 15 of a wave).
LCMA_DEV float block_amax(float m) {
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) m = __builtin_fmaxf(m, __shfl_xor(m, d, 16));
    return m;
}

LCMA_DEV void widen_bf16(u32x4 raw, float (&out)[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        out[2 * e] = __builtin_bit_cast(float, raw[e] << 16);
        out[2 * e + 1] = __builtin_bit_cast(float, raw[e] & 0xffff0000u);
    }
}

// One thread: 8 consecutive k of one row; 16 threads: one scale block; a work-group of 256: 16 rows x 128 k.
// grid.x: row groups of 16, grid.y: scale blocks along K.  HBM-bound: reads 2 bytes and writes 1 + 1/128 per element.
LCMA_DEV void fp8_quantize_rows_tile(const Fp8QuantParams &p) {
    const auto rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.X), 0, (int)p.x_bytes, 0x00020000);
    const auto rq = __builtin_amdgcn_make_buffer_rsrc(p.Q, 0, (int)p.q_bytes, 0x00020000);
    const auto rs = __builtin_amdgcn_make_buffer_rsrc(p.S, 0, (int)p.s_bytes, 0x00020000);
    // (work-groups that start together cover consecutive 128-element blocks of the same 16 rows)
    const uint32_t row = blockIdx.y * 16 + threadIdx.x / 16, kb = blockIdx.x, c = threadIdx.x % 16;
    if ((int)row >= p.rows) return;
    const uint32_t colb = kb * 256 + c * 16; // byte column in X
    float v[8];
    widen_bf16(__builtin_amdgcn_raw_buffer_load_b128(rx, (int)(colb < p.k_row_b ? row * p.ldx_b + colb : p.x_bytes), 0, 0), v);
    float m = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(v[e]));
    const int sb = scale_byte_of(block_amax(m));
    const u32x2 q = quantize8(v, sb - 127);
    __builtin_amdgcn_raw_buffer_store_b64(q, rq, (int)(row * p.ldq_b + kb * 128 + c * 8), 0, 0);
    if (c == 0) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sb, rs, (int)(row * p.lds_b + kb), 0, 0);
}

// Combine A / Combine B for N x K weights with the quantisation fused in.  CH (generated): NB raw blocks with
// b_j(t) (block row) and b_l(t) (block column along K) and comb(in, r), the signed fp32 sum of product r in
// ascending block order.  Same thread layout as above; every thread forms its 8 elements of all NP planes.
template <class CH> LCMA_DEV void fp8_combine_quantize_tile(const Fp8QuantParams &p) {
    const auto rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.X), 0, (int)p.x_bytes, 0x00020000);
    const auto rq = __builtin_amdgcn_make_buffer_rsrc(p.Q, 0, (int)p.q_bytes, 0x00020000);
    const auto rs = __builtin_amdgcn_make_buffer_rsrc(p.S, 0, (int)p.s_bytes, 0x00020000);
    // (work-groups that start together cover consecutive 128-element blocks of the same 16 rows)
    const uint32_t row = blockIdx.y * 16 + threadIdx.x / 16, kb = blockIdx.x, c = threadIdx.x % 16;
    if ((int)row >= p.rows) return;
    u32x4 in[CH::NB]; // as loaded; widened where a sum uses them (see forget_derived)
#pragma unroll
    for (int t = 0; t < CH::NB; ++t) {
        // blocks are cut from the matrix padded (virtually, with zeros) to whole planes: the block steps are those of
        // the padded sizes, so rows past the last row fall outside the extent (read as zero by the range check) and
        // columns past K are sent there
        const uint32_t colb = (uint32_t)CH::b_l(t) * p.x_bcol + kb * 256 + c * 16;
        const uint32_t off = colb < p.k_row_b ? (uint32_t)CH::b_j(t) * p.x_brow + row * p.ldx_b + colb : p.x_bytes;
        in[t] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0);
    }
    for_each_const<CH::NP>([&](auto rc_) {
        constexpr int r = decltype(rc_)::value;
        forget_derived(in);
        float v[8], m = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float col[CH::NB];
#pragma unroll
            for (int t = 0; t < CH::NB; ++t) col[t] = Elem<BF16>::get(in[t], e);
            v[e] = CH::comb(col, r);
            m = __builtin_fmaxf(m, __builtin_fabsf(v[e]));
        }
        const int sb = scale_byte_of(block_amax(m));
        const u32x2 q = quantize8(v, sb - 127);
        __builtin_amdgcn_raw_buffer_store_b64(q, rq, (int)(row * p.ldq_b + kb * 128 + c * 8), (int)(r * p.q_plane), 0);
        if (c == 0) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sb, rs, (int)(row * p.lds_b + kb), (int)(r * p.s_plane), 0);
    });
}

} // namespace lcma
