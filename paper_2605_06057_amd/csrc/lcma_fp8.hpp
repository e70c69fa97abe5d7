// FP8 path for gfx950 (CDNA4): E4M3 operands with one power-of-two scale per 1 x 128 block along K.
//
// The paper's FP8 workflow (Sec. 4.1, experimental setup: bf16 operands quantised to FP8 E4M3 with 1 x 128 block-wise
// scaling; Sec. 4.3: the quantisation fused into the Combine A stage) on MI355X's own terms: a scale is 2^e stored as
// the byte e + 127 (the E8M0 scale type), which the scaled matrix instruction v_mfma_scale_f32_32x32x64_f8f6f4 applies
// in hardware, so the block-scaled product costs no vector instruction per element and accumulates across the K/128
// blocks in one set of fp32 registers.  e is the smallest integer with amax <= 448 * 2^e (0 for an all-zero block):
// dividing by 2^e is exact, the one rounding is the conversion to E4M3 (nearest, ties to even).
//
// Three kinds of kernel:
//   quantize_rows        bf16 matrix -> codes + scale bytes (the plain workflow, and static weights);
//   combine_quantize     Combine A (Eq. 3) or Combine B for N x K weights (Eq. 4) with the quantisation fused in: the
//                        signed sums are formed in fp32 in ascending block order (generated code) and leave the kernel
//                        as E4M3 planes with their scales;
//   fp8_gemm             C = A x W^T on codes and scales (Eq. 5 on the dequantised operands), optionally batched over
//                        the R planes of a scheme (the GEMM stage of Algorithm 1).
// Layouts: code matrices are row-major and k-contiguous (A: M x K, W: N x K), one byte per element; a scale matrix
// has one row per row of codes and K/128 bytes per row, the row pitch padded to a multiple of 4 bytes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_device.hpp"

namespace lcma {

typedef int i32x8 __attribute__((ext_vector_type(8)));
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
    const uint32_t row = blockIdx.x * 16 + threadIdx.x / 16, kb = blockIdx.y, c = threadIdx.x % 16;
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
    const uint32_t row = blockIdx.x * 16 + threadIdx.x / 16, kb = blockIdx.y, c = threadIdx.x % 16;
    if ((int)row >= p.rows) return;
    float in[CH::NB][8];
#pragma unroll
    for (int t = 0; t < CH::NB; ++t) {
        // blocks are cut from the matrix padded (virtually, with zeros) to whole planes: the block steps are those of
        // the padded sizes, so rows past the last row fall outside the extent (read as zero by the range check) and
        // columns past K are sent there
        const uint32_t colb = (uint32_t)CH::b_l(t) * p.x_bcol + kb * 256 + c * 16;
        const uint32_t off = colb < p.k_row_b ? (uint32_t)CH::b_j(t) * p.x_brow + row * p.ldx_b + colb : p.x_bytes;
        widen_bf16(__builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0), in[t]);
    }
#pragma unroll
    for (int r = 0; r < CH::NP; ++r) {
        float v[8], m = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float col[CH::NB];
#pragma unroll
            for (int t = 0; t < CH::NB; ++t) col[t] = in[t][e];
            v[e] = CH::comb(col, r);
            m = __builtin_fmaxf(m, __builtin_fabsf(v[e]));
        }
        const int sb = scale_byte_of(block_amax(m));
        const u32x2 q = quantize8(v, sb - 127);
        __builtin_amdgcn_raw_buffer_store_b64(q, rq, (int)(row * p.ldq_b + kb * 128 + c * 8), (int)(r * p.q_plane), 0);
        if (c == 0) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sb, rs, (int)(row * p.lds_b + kb), (int)(r * p.s_plane), 0);
    }
}

// ---------------------------------------------------------------- block-scaled GEMM on codes
// One work-group: a TM x TN tile of C (of one plane when BATCH); y walks the K/128 scale blocks.  Per step the
// 128-byte rows of both operands travel global -> registers -> LDS (16-byte chunks, XOR-swizzled), a wave reads its
// fragments (lane: row lane % 32, 32 consecutive k at (lane / 32) * 32 of a 64-k half) and issues two scaled MFMAs per
// 32 x 32 tile with the E8M0 bytes of its rows; the accumulators hold the block-scaled sum directly.
// OUT: BF16 (C of the plain workflow) or F16 (the planes H_r of Algorithm 1).
template <int TM, int TN, int WGM, int WGN, bool BATCH, class OUT> struct Fp8Gemm {
    static constexpr int NT = 64 * WGM * WGN, WM = TM / WGM, WN = TN / WGN, NMI = WM / 32, NNI = WN / 32;
    static constexpr int ROW = 128, A_STAGE = TM * ROW, B_STAGE = TN * ROW, STAGE = A_STAGE + B_STAGE;
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int QA = TM * 8 / NT, QB = TN * 8 / NT;
    static_assert(TM * 8 % NT == 0 && TN * 8 % NT == 0 && WM % 32 == 0 && WN % 32 == 0, "tile and wave grid");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");

    // 128-byte rows: two rows per 256-byte bank window; 16 consecutive rows at one chunk column spread over the 16
    // chunk positions of a window
    static LCMA_DEV constexpr int swz(int row, int c) { return c ^ ((row >> 1) & 7); }

    static LCMA_DEV void run(const Fp8GemmParams &p, LCMA_LDS char *lds) {
        const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w / WGN, wn = w % WGN;
        const int l32 = lane & 31, lh = lane >> 5;
        // tile order: a contiguous run of tiles per XCD (work-groups are dealt to the 8 XCDs round-robin), tiles run
        // down x inside column panels; batched: product-major, so that concurrent work-groups share r
        const int tiles = p.nx * p.nz, total = (int)gridDim.x;
        int id = blockIdx.x;
        const int per = total >> 3;
        if (id < (per << 3)) id = (id & 7) * per + (id >> 3);
        int plane = 0;
        if constexpr (BATCH) {
            plane = id / tiles;
            id -= plane * tiles;
        }
        const int pw = p.panel, full = (p.nz / pw) * pw * p.nx;
        int x, z;
        if (id < full) {
            const int pi = id / (pw * p.nx), rem = id - pi * (pw * p.nx);
            x = rem / pw;
            z = pi * pw + rem % pw;
        } else {
            const int w2 = p.nz - (p.nz / pw) * pw, rem = id - full;
            x = rem / w2;
            z = (p.nz / pw) * pw + rem % w2;
        }
        const auto ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.A), 0, (int)p.a_bytes, 0x00020000);
        const auto rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.B), 0, (int)p.b_bytes, 0x00020000);
        const auto rsa = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.SA), 0, (int)p.sa_bytes, 0x00020000);
        const auto rsb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.SB), 0, (int)p.sb_bytes, 0x00020000);
        const auto rc = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)p.c_bytes, 0x00020000);
        const uint32_t a_base = (uint32_t)plane * p.a_plane + (uint32_t)x * TM * p.lda_b;
        const uint32_t b_base = (uint32_t)plane * p.b_plane + (uint32_t)z * TN * p.ldb_b;

        uint32_t a_voff[QA], a_lds[QA], b_voff[QB], b_lds[QB];
#pragma unroll
        for (int q = 0; q < QA; ++q) {
            const int idx = q * NT + tid, row = idx >> 3, c = idx & 7;
            a_voff[q] = (uint32_t)row * p.lda_b + c * 16;
            a_lds[q] = row * ROW + swz(row, c) * 16;
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int idx = q * NT + tid, row = idx >> 3, c = idx & 7;
            b_voff[q] = (uint32_t)row * p.ldb_b + c * 16;
            b_lds[q] = A_STAGE + row * ROW + swz(row, c) * 16;
        }
        // fragment addresses: chunk pair (2 j, 2 j + 1) of half kk, j = lane / 32
        uint32_t a_frag[2][2], b_frag[2][2];
        const int ar = wm * WM + l32, br = wn * WN + l32;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                a_frag[kk][j] = ar * ROW + swz(ar, kk * 4 + lh * 2 + j) * 16;
                b_frag[kk][j] = A_STAGE + br * ROW + swz(br, kk * 4 + lh * 2 + j) * 16;
            }
        // scale bytes of this lane's rows: one dword holds four consecutive K blocks
        const uint32_t sa_base = (uint32_t)plane * p.sa_plane + (uint32_t)(x * TM + ar) * p.lsa_b;
        const uint32_t sb_base = (uint32_t)plane * p.sb_plane + (uint32_t)(z * TN + br) * p.lsb_b;
        uint32_t sa_cur[NMI], sa_nxt[NMI], sb_cur[NNI], sb_nxt[NNI];
        auto load_scales = [&](int g, uint32_t (&sa)[NMI], uint32_t (&sb)[NNI]) {
#pragma unroll
            for (int mi = 0; mi < NMI; ++mi)
                sa[mi] = __builtin_amdgcn_raw_buffer_load_b32(rsa, (int)(sa_base + (uint32_t)mi * 32 * p.lsa_b + g * 4), 0, 0);
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni)
                sb[ni] = __builtin_amdgcn_raw_buffer_load_b32(rsb, (int)(sb_base + (uint32_t)ni * 32 * p.lsb_b + g * 4), 0, 0);
        };

        f32x16 acc[NMI][NNI];
#pragma unroll
        for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni) zero(acc[mi][ni]);

        u32x4 rega[QA], regb[QB];
        auto issue = [&](int y) {
#pragma unroll
            for (int q = 0; q < QA; ++q) rega[q] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_voff[q], (int)(a_base + (uint32_t)y * ROW), 0);
#pragma unroll
            for (int q = 0; q < QB; ++q) regb[q] = __builtin_amdgcn_raw_buffer_load_b128(rb, (int)b_voff[q], (int)(b_base + (uint32_t)y * ROW), 0);
        };
        auto store = [&](int st) {
#pragma unroll
            for (int q = 0; q < QA; ++q) *(LCMA_LDS u32x4 *)(lds + st * STAGE + a_lds[q]) = rega[q];
#pragma unroll
            for (int q = 0; q < QB; ++q) *(LCMA_LDS u32x4 *)(lds + st * STAGE + b_lds[q]) = regb[q];
        };
        auto frag = [&](uint32_t off0, uint32_t off1) {
            const u32x4 lo = *(LCMA_LDS u32x4 *)(lds + off0), hi = *(LCMA_LDS u32x4 *)(lds + off1);
            return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        };
        const int ny = p.ny, last = ny - 1;
        issue(0);
        load_scales(0, sa_cur, sb_cur);
        load_scales(1, sa_nxt, sb_nxt);
        auto step = [&](int y, int st) { // st is a literal at both call sites
            store(st);
            issue(y + 1 < ny ? y + 1 : last); // past the end: the last tile again, unused
            if ((y & 3) == 0 && y > 0) {      // uniform: the scales of the next four blocks arrive a group ahead
#pragma unroll
                for (int mi = 0; mi < NMI; ++mi) sa_cur[mi] = sa_nxt[mi];
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni) sb_cur[ni] = sb_nxt[ni];
                load_scales((y >> 2) + 1, sa_nxt, sb_nxt);
            }
            __syncthreads();
            const int sh = (y & 3) * 8;
            int sa[NMI], sb[NNI];
#pragma unroll
            for (int mi = 0; mi < NMI; ++mi) sa[mi] = (int)((sa_cur[mi] >> sh) & 0xffu);
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni) sb[ni] = (int)((sb_cur[ni] >> sh) & 0xffu);
            const uint32_t sbase = st * STAGE;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                i32x8 a[NMI], b[NNI];
#pragma unroll
                for (int mi = 0; mi < NMI; ++mi)
                    a[mi] = frag(sbase + a_frag[kk][0] + mi * 32 * ROW, sbase + a_frag[kk][1] + mi * 32 * ROW);
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni)
                    b[ni] = frag(sbase + b_frag[kk][0] + ni * 32 * ROW, sbase + b_frag[kk][1] + ni * 32 * ROW);
#pragma unroll
                for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NNI; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[mi], b[ni], acc[mi][ni], 0, 0, 0, sa[mi], 0, sb[ni]);
            }
        };
        int y = 0;
        for (; y + 1 < ny; y += 2) {
            step(y, 0);
            step(y + 1, 1);
        }
        if (y < ny) step(y, 0);

        // Epilogue.  Accumulator value v of tile (mi, ni) is row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32: a
        // lane's values lie in one column.  Each wave therefore passes one 32-row strip of its tile at a time through a
        // private piece of LDS (the stages are free now) and writes it out as 16-byte vectors, whole 128-byte lines.
        // The scalar-offset field of these stores stays a literal zero (everything is in the vector offset): the
        // compiler keeps a following vector write at a distance from a store of more than 8 bytes only then.
        constexpr int PITCH = WN * 2 + 16, CPRW = WN * 2 / 16, NIT = 32 * CPRW / 64;
        static_assert(NT / 64 * 32 * PITCH <= LDS_BYTES, "the strips of all waves fit the stage buffers");
        const uint32_t c_base = (uint32_t)plane * p.c_plane + (uint32_t)x * TM * p.ldc_b + (uint32_t)z * TN * 2;
        LCMA_LDS char *strip = lds + w * (32 * PITCH);
        __syncthreads(); // every wave is done reading the stages
#pragma unroll
        for (int mi = 0; mi < NMI; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    *(LCMA_LDS uint16_t *)(strip + ((v >> 2) * 8 + 4 * lh + (v & 3)) * PITCH + (ni * 32 + l32) * 2) =
                        (uint16_t)Round<OUT>::run(acc[mi][ni][v]);
            __syncthreads();
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int idx = it * 64 + lane, row = idx / CPRW, ch = idx % CPRW;
                const u32x4 v = *(LCMA_LDS u32x4 *)(strip + row * PITCH + ch * 16);
                const uint32_t colb = (uint32_t)(wn * WN) * 2 + ch * 16; // byte column inside the tile
                // a vector past N goes to the end of the extent and is dropped (N is a whole number of vectors); rows
                // past M fall outside the extent by themselves
                const uint32_t off = ((uint32_t)z * TN * 2 + colb < p.n_row_b)
                                         ? c_base + (uint32_t)(wm * WM + mi * 32 + row) * p.ldc_b + colb
                                         : p.c_bytes;
                __builtin_amdgcn_raw_buffer_store_b128(v, rc, (int)off, 0, 0);
            }
            __syncthreads();
        }
    }
};

} // namespace lcma
