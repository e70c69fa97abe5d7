// Device-side building blocks of the fused LCMA kernel for gfx950 (CDNA4, 64-wide waves).
//
// One work-group (4 or 8 waves) owns one GROUP in the sense of the paper's Group-Parallel
// Optimization (Sec. 3.2, Algorithm 2): the tile at coordinate (x, z) of every block of C.
// The R products of the scheme are cut into CHUNKS.  For a chunk the work-group walks y
// (the K/k direction) and multiplies with MFMA into one fp32 accumulator tile per product
// (Eq. 5); after the chunk the generated code applies W (Eq. 6) in fp32 registers.  Nothing
// but C is ever written to device memory.  Two dataflows form the operands of Eq. 3 / Eq. 4:
//   staged combine    the tiles A_{i,l}[x,y], B_{l,j}[y,z] the chunk needs are loaded, combined
//                     in registers and the combined tiles At_r, Bt_r written to LDS;
//   fragment combine  the raw (converted) tiles are written to LDS and every wave combines the
//                     MFMA fragments it reads (all R products advance together; the fast path).
// With the offline Combine-B stage the right operands come from memory ready-made and go to
// LDS untouched.  Everything that depends on U, V, W is straight-line generated code
// (Sec. 3.1, coefficients as compile-time constants); this header is scheme-agnostic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "lcma_params.h"

namespace lcma {

// Cache-policy operand of the buffer builtins for the stores of data that no later stage re-reads from the caches: the
// products H_r that the batched GEMM of Algorithm 1 hands to Combine H, and C.  Bit 1 = non-temporal: such lines are
// the first to leave the L2 and the Infinity Cache, instead of displacing the planes At_r / Bt_r that the work-groups of
// the batched GEMM read again and again.  Measured on the whole of Algorithm 1, bf16: +4 % at 8192 x 14336 x 4096, +6 %
// at 4096^3.  Loads are NOT given the policy: on the inputs A and B it makes Combine A / Combine B 15 % (large shape)
// to 90 % (4096^3) slower, on the planes H_r in Combine H it gains 0.3 % for fp16 planes and loses 4 % for fp32 planes.
constexpr int kStreamed = 2;


typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define LCMA_LDS __attribute__((address_space(3)))
#define LCMA_DEV __device__ __forceinline__
#ifndef LCMA_FP32_GROUP
#define LCMA_FP32_GROUP 2 // products whose fp32 MFMA chains are interleaved
#endif

// ---------------------------------------------------------------- element types
// ES: bytes per element, CH: elements per 16-byte chunk, vec: what the combination code adds.
struct F32 {
    static constexpr int ES = 4, CH = 4;
    using vec = f32x4;
};
struct F16 {
    static constexpr int ES = 2, CH = 8;
    using vec = f16x8;
};
struct BF16 { // opaque in registers: only moved, never added
    static constexpr int ES = 2, CH = 8;
    using vec = u32x4;
};

// Storage type -> type the combinations are formed and multiplied in.
template <class IN, class CT> struct Convert;
template <class T> struct Convert<T, T> {
    static LCMA_DEV typename T::vec run(u32x4 raw) { return __builtin_bit_cast(typename T::vec, raw); }
};
// bf16 -> fp16: widen each half to fp32 (a shift or a mask), then pack two to fp16.  Exact for
// magnitudes in [2^-14, 65504] because bf16 carries 8 significant bits and fp16 carries 11.
template <> struct Convert<BF16, F16> {
    static LCMA_DEV f16x8 run(u32x4 raw) {
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __builtin_bit_cast(float, raw[i] << 16);
            const float hi = __builtin_bit_cast(float, raw[i] & 0xffff0000u);
            out[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
        }
        return __builtin_bit_cast(f16x8, out);
    }
};

// Sums of three or more fp16 terms are formed in fp32 and rounded once (nearest-even); two-term
// sums are already rounded once by the packed fp16 add.  Other vector types add in place.
typedef float f32x8 __attribute__((ext_vector_type(8)));
template <class V> struct Wide {
    static LCMA_DEV V up(const V &v) { return v; }
    static LCMA_DEV V down(const V &v) { return v; }
};
template <> struct Wide<f16x8> {
    static LCMA_DEV f32x8 up(const f16x8 &v) { return __builtin_convertvector(v, f32x8); }
    static LCMA_DEV f16x8 down(const f32x8 &v) { return __builtin_convertvector(v, f16x8); }
    // what rounding v to fp16 loses, as fp16
    static LCMA_DEV f16x8 residual(const f32x8 &v) { return down(v - up(down(v))); }
};

// Element-wise add / subtract of the vectors the combinations are formed on.  A packed fp16
// subtraction is written as fma(b, -1, a) with the -1 hidden from the optimiser: the compiler
// otherwise splits a packed fp16 subtraction into two scalar subtractions and a pack per dword.
// (No instruction is written by hand, so hazard handling stays with the compiler.)
template <class V> LCMA_DEV V vadd(const V &a, const V &b) { return a + b; }
template <class V> LCMA_DEV V vsub(const V &a, const V &b) { return a - b; }
LCMA_DEV f16x8 vsub(const f16x8 &a, const f16x8 &b) {
    uint32_t m = 0xBC00BC00u; // (-1.0h, -1.0h)
    asm("" : "+v"(m)); // not volatile: identical copies merge into one
    const u32x4 m4 = {m, m, m, m};
    return __builtin_elementwise_fma(b, __builtin_bit_cast(f16x8, m4), a);
}

// fp32 accumulator -> storage element (one rounding, nearest-even), as raw bits.
template <class IN> struct Round;
template <> struct Round<F32> {
    static LCMA_DEV uint32_t run(float v) { return __builtin_bit_cast(uint32_t, v); }
};
template <> struct Round<F16> {
    static LCMA_DEV uint32_t run(float v) { return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v); }
};
template <> struct Round<BF16> {
    static LCMA_DEV uint32_t run(float v) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)v); }
};

// ---------------------------------------------------------------- tile configuration
// TM x TN: tile of one block product owned by the work-group; TK: depth per y step;
// WGM x WGN: wave grid (4 waves); NSA / NSB: A-side / B-side tiles resident per LDS stage;
// PIPE: 0 staging in one phase before the barrier, 2 staging spread over the MFMA phase
//       (fragment-combine kernels only);
// FC: 0 = combinations are formed while staging and LDS holds At_r, Bt_r;
//     1 = LDS holds the raw (converted) blocks and every wave forms the combinations on the
//         MFMA fragments it has read ("fragment combine");
// STAGES: LDS stages (2, or 3 with PIPE 2 and FC: the first fragments of the next step are then read
//         before the barrier that ends the step);
// PB: 1 = the B operand is the output of the offline Combine-B stage (Eq. 4 done once for static
//         weights): R planes of (N/n) x (K/k) elements of the compute type, k-contiguous.  Tiles of the
//         right operands Bt_r go to LDS as they are (no conversion, transposition or addition) and
//         only the A side is combined on fragments;
// DL: 1 (with PB) = tiles travel from memory straight into LDS (buffer loads with the LDS bit: no
//         staging registers, no LDS write instructions); the raw A blocks then sit in LDS in the
//         storage type and are converted on the fragments;
// TB: 1 = B is given as the N x K matrix W with W[n][k] = B[k][n] (the layout of a linear layer's
//         weight): its rows are k-contiguous like those of A, so its tiles are staged exactly like
//         A's (16-byte loads, no transposition);
// PA: 1 (staged loop, with PB) = the left operands At_r come from memory ready-made as well (the
//         stand-alone Combine-A stage of Algorithm 2): R planes of (M/m) x (K/k) elements of the
//         compute type.  The kernel is then Algorithm 2's fused GEMM + Combine-H stage alone;
// BATCH: 1 (plain kernels on planes) = the grid covers R independent products: work-group id / tiles
//         per product selects the plane of A, B and C (the batched GEMM stage of Algorithm 1).
//
// LDS layout of a stage: NSA tiles [TM rows][TK] then NSB tiles [TN rows][TK], both k-contiguous,
// 16-byte chunks XOR-swizzled inside a row.  B arrives n-contiguous from memory and is transposed
// in registers while it is staged, so that both MFMA operands are read with 16-byte LDS loads
// (measured on MI355X: ds_read_b128 ~260 B/clk/CU, the transposing ds_read_b64_tr_b16 ~70).
template <class IN_, class CT_, int TM_, int TN_, int TK_, int WGM_, int WGN_, int NSA_, int NSB_, int PIPE_ = 0,
          int FC_ = 0, int STAGES_ = 2, int PB_ = 0, int DL_ = 0, int TB_ = 0, int PA_ = 0, int BATCH_ = 0>
struct Tile {
    static constexpr int PIPE = PIPE_, FC = FC_, PB = PB_, DL = DL_, TB = TB_, PA = PA_, BATCH = BATCH_;
    static_assert(!PA_ || (PB_ && !FC_), "ready-made left operands: staged loop, both sides from planes");
    static_assert(!TB_ || !PB_, "a prepared operand has one layout only");
    static_assert(!DL_ || PB_ || (TB_ && FC_ && PIPE_ == 2 && STAGES_ == 3 && std::is_same_v<IN_, CT_>),
                  "direct loads need operands that go to LDS untouched on both sides: prepared B, or k-contiguous B "
                  "in a storage type that is multiplied as it is (three stages, fragment-combine loop)");
    static_assert(!PB_ || (FC_ && PIPE_ == 2 && STAGES_ == 2) || (!FC_ && PIPE_ == 0),
                  "prepared B: the interleaved fragment-combine loop or the staged loop");
    using IN = IN_;
    using CT = CT_;
    static_assert(IN::ES == CT::ES, "conversion must keep the element size");
    static constexpr int TM = TM_, TN = TN_, TK = TK_, WGM = WGM_, WGN = WGN_;
    static constexpr int NSA = NSA_, NSB = NSB_, STAGES = STAGES_;
    static constexpr int ES = CT::ES, CH = CT::CH;
    static constexpr int NT = 64 * WGM * WGN;
    static constexpr int WM = TM / WGM, WN = TN / WGN;
    static constexpr int NMI = WM / 32, NNI = WN / 32;
    static constexpr int KSTEP = (ES == 2) ? 16 : 8; // k covered by one fragment read
    static constexpr int NKK = TK / KSTEP;
    static constexpr int CPR = TK / CH;        // 16-byte chunks per LDS row
    static constexpr int ROW = TK * ES;        // LDS row pitch in bytes
    static constexpr int NCHK_A = TM * CPR;    // A is staged one 16-byte chunk per thread and step
    static constexpr int QA = (NCHK_A + NT - 1) / NT;
    // B (K x N) is staged in units: 16-bit: a column pair x 8 consecutive k (8 dword loads -> 2 chunks);
    // fp32: one column x 4 consecutive k (4 dword loads -> 1 chunk).  Given as N x K a unit is one
    // 16-byte chunk of a row, as for A.
    static constexpr int BW = (ES == 2) ? 8 : 4;   // dword loads per unit
    static constexpr int BH = TB ? 1 : BW / 4;     // 16-byte register vectors per unit
    static constexpr int BCOLS = (ES == 2) ? TN / 2 : TN;
    static constexpr int NU_B = TB ? TN * CPR : BCOLS * CPR;
    static constexpr int QB = (NU_B + NT - 1) / NT;
    static constexpr int NCHK_BP = TN * CPR;   // 16-byte chunks of one tile of a prepared right operand
    static constexpr int QBP = (NCHK_BP + NT - 1) / NT;
    static constexpr int A_SLOT = TM * ROW, B_SLOT = TN * ROW;
    static constexpr int A_STAGE = NSA * A_SLOT, B_STAGE = NSB * B_SLOT;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int LDS_BYTES = STAGES * STAGE;
    static_assert(NT == 256 || NT == 512, "four or eight waves per work-group");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && TK % KSTEP == 0, "MFMA 32x32 tiling");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");

    struct Acc {
        f32x16 v[NMI][NNI];
    };

    // XOR swizzle of the chunk index: a fragment read touches 16 consecutive rows at one chunk
    // column; spread them over the 16 chunk positions of a 256-byte bank window.
    static LCMA_DEV constexpr int swz(int row, int c) {
        constexpr int rpw = (CPR >= 16) ? 1 : 16 / CPR; // rows per 256-byte window
        constexpr int mask = (CPR >= 16) ? 15 : CPR - 1;
        return c ^ ((row / rpw) & mask);
    }
};

// In the fragment-combine loop a wave raises its issue priority while it issues MFMA instructions, so
// that, of the waves sharing a SIMD, the one with a multiplication ready goes first and the matrix
// pipe does not idle behind another wave's vector work.  Measured in one run, with and without: +7%
// on the fp32 Strassen kernel, +1% on the 16-bit ones; the staged, plain and prepared-B loops lose
// 1-3% with it and do not use it.
#ifndef LCMA_SETPRIO
#define LCMA_SETPRIO 1
#endif
#ifndef LCMA_EPILOGUE_LDS
#define LCMA_EPILOGUE_LDS 1 // 16-bit C tiles leave through LDS as 16-byte stores (0: 2-byte stores, for comparison)
#endif
LCMA_DEV void mfma_priority(bool on) {
#if LCMA_SETPRIO > 0
    if (on) __builtin_amdgcn_s_setprio(LCMA_SETPRIO);
    else __builtin_amdgcn_s_setprio(0);
#endif
}

LCMA_DEV void zero(f32x16 &v) {
#pragma unroll
    for (int e = 0; e < 16; ++e) v[e] = 0.f;
}
template <class ACC> LCMA_DEV void zero_acc(ACC &a) {
#pragma unroll
    for (auto &row : a.v)
#pragma unroll
        for (auto &t : row) zero(t);
}

// Eq. 6 on accumulator tiles: c = w * h and c += w * h (w is a literal, +-1 in the usual schemes).
template <class ACC> LCMA_DEV void acc_set(ACC &c, const ACC &h, float w) {
#pragma unroll
    for (int a = 0; a < (int)(sizeof(c.v) / sizeof(c.v[0])); ++a)
#pragma unroll
        for (int b = 0; b < (int)(sizeof(c.v[0]) / sizeof(c.v[0][0])); ++b) c.v[a][b] = h.v[a][b] * w;
}
template <class ACC> LCMA_DEV void acc_add(ACC &c, const ACC &h, float w) {
#pragma unroll
    for (int a = 0; a < (int)(sizeof(c.v) / sizeof(c.v[0])); ++a)
#pragma unroll
        for (int b = 0; b < (int)(sizeof(c.v[0]) / sizeof(c.v[0][0])); ++b) c.v[a][b] += h.v[a][b] * w;
}

// One MFMA step.  16-bit: a, b hold 8 consecutive k each.  fp32: 4 consecutive k each, issued as
// four 32x32x2 instructions (instruction t multiplies k = 4*(lane/32) + t on both sides).
template <class CT> struct Mma;
template <> struct Mma<F16> {
    using frag = f16x8;
    static constexpr int SUB = 1;
    static LCMA_DEV void run_sub(const frag &a, const frag &b, f32x16 &c, int) { run(a, b, c); }
    static LCMA_DEV void run(const frag &a, const frag &b, f32x16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<BF16> {
    using frag = bf16x8;
    static constexpr int SUB = 1;
    static LCMA_DEV void run_sub(const frag &a, const frag &b, f32x16 &c, int) { run(a, b, c); }
    static LCMA_DEV void run(const frag &a, const frag &b, f32x16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<F32> {
    using frag = f32x4;
    static constexpr int SUB = 4; // instructions per fragment pair
    static LCMA_DEV void run_sub(const frag &a, const frag &b, f32x16 &c, int t) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], c, 0, 0, 0);
    }
    static LCMA_DEV void run(const frag &a, const frag &b, f32x16 &c) {
#pragma unroll
        for (int t = 0; t < 4; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------- per-work-group context
template <class T> struct Ctx {
    using IN = typename T::IN;
    using CT = typename T::CT;
    using V = typename CT::vec;
    using Frag = typename Mma<CT>::frag;

    const Params &p;
    LCMA_LDS char *lds;
    __amdgpu_buffer_rsrc_t ra, rb, rc;
    int lane, wm, wn;
    uint32_t a_group, b_group, c_group; // byte offsets of this group's tile inside a block
    uint32_t n_group;                   // first column n of the tile inside a block, in bytes of a row of C
    uint32_t a_voff[T::QA], b_voff[T::QB];
    uint32_t a_lds[T::QA], b_lds[T::QB], b_lds1[T::QB]; // b_lds1: second LDS row of a 16-bit B unit
    uint32_t a_frag[T::NKK], b_frag[T::NKK];
    uint32_t c_voff; // byte offset of this lane's first output element inside the tile
    uint32_t c_colb; // byte column of that element inside a block of C (for the N bound)
    uint32_t b_colb[T::QB]; // position n (in bytes of a row of C) inside a block of the unit staged by this thread
    uint32_t bp_voff[T::QBP], bp_lds[T::QBP]; // staged kernels with prepared B: chunks of a Bt_r tile

    LCMA_DEV Ctx(const Params &p_, LCMA_LDS char *lds_) : p(p_), lds(lds_) {
        ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.A), 0, (int)p.a_bytes, 0x00020000);
        rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.B), 0, (int)p.b_bytes, 0x00020000);
        rc = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)p.c_bytes, 0x00020000);
        const int tid = threadIdx.x;
        lane = tid & 63;
        const int w = tid >> 6;
        wm = w / T::WGN;
        wn = w % T::WGN;

        // Tile order.  Hardware deals work-groups to the 8 XCDs round-robin; give each XCD
        // a contiguous run of tiles so that its private L2 sees neighbouring tiles.  Tiles
        // run down x inside column panels of `panel` z-tiles.
        const int tiles = p.nx * p.nz;
        const int total = T::BATCH ? (int)gridDim.x : tiles;
        int id = blockIdx.x;
        const int per = total >> 3;
        if (id < (per << 3)) id = (id & 7) * per + (id >> 3);
        int plane = 0;
        if constexpr (T::BATCH) {
            if (p.batch_order == 0) {
                plane = id / tiles;
                id -= plane * tiles;
            } else {
                const int R = total / tiles;
                plane = id % R;
                id /= R;
            }
        }
        const int pw = p.panel;
        const int full = (p.nz / pw) * pw * p.nx; // tiles inside full-width panels
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
        a_group = (uint32_t)x * T::TM * p.lda_b;
        b_group = (T::PB || T::TB) ? (uint32_t)z * T::TN * p.ldb_b : (uint32_t)z * T::TN * T::ES;
        c_group = (uint32_t)x * T::TM * p.ldc_b + (uint32_t)z * T::TN * T::ES;
        n_group = (uint32_t)z * T::TN * T::ES;
        if constexpr (T::BATCH) { // plane strides sit where the block-row steps of a scheme would
            a_group += (uint32_t)plane * p.a_brow;
            b_group += (uint32_t)plane * p.b_brow;
            c_group += (uint32_t)plane * p.c_brow;
        }

#pragma unroll
        for (int q = 0; q < T::QA; ++q) {
            // a tile smaller than the work-group is staged twice by threads that wrap around
            // (same data to the same address), which keeps the pipeline free of branches
            const int id2 = (q * T::NT + tid) % T::NCHK_A;
            const int row = id2 / T::CPR, c = id2 % T::CPR;
            a_voff[q] = (uint32_t)row * p.lda_b + c * 16;
            a_lds[q] = row * T::ROW + T::swz(row, c) * 16;
        }
#pragma unroll
        for (int q = 0; q < T::QB; ++q) {
            // consecutive lanes take consecutive columns (coalesced dword loads along a row of B)
            const int u = (q * T::NT + tid) % T::NU_B;
            if constexpr (T::TB) { // rows n of the tile, k-contiguous: as for A
                const int row = u / T::CPR, c = u % T::CPR;
                b_voff[q] = (uint32_t)row * p.ldb_b + c * 16;
                b_colb[q] = (uint32_t)(z * T::TN + row) * T::ES;
                b_lds[q] = T::A_STAGE + row * T::ROW + T::swz(row, c) * 16;
                b_lds1[q] = 0;
            } else {
                const int col = u % T::BCOLS, g = u / T::BCOLS; // g: group of CH consecutive k
                const int row = (T::ES == 2) ? 2 * col : col;   // LDS row = column n of the tile
                b_voff[q] = (uint32_t)(g * T::CH) * p.ldb_b + col * 4;
                b_colb[q] = (uint32_t)z * T::TN * T::ES + col * 4;
                b_lds[q] = T::A_STAGE + row * T::ROW + T::swz(row, g) * 16;
                b_lds1[q] = T::A_STAGE + (row + 1) * T::ROW + T::swz(row + 1, g) * 16;
            }
        }
#pragma unroll
        for (int q = 0; q < T::QBP; ++q) {
            const int id2 = (q * T::NT + tid) % T::NCHK_BP;
            const int row = id2 / T::CPR, c = id2 % T::CPR;
            bp_voff[q] = (uint32_t)row * p.ldb_b + c * 16;
            bp_lds[q] = T::A_STAGE + row * T::ROW + T::swz(row, c) * 16;
        }
        // Fragment addresses.  Operand of the 32x32 MFMA: lane holds row lane%32 and the
        // (lane/32)-th group of consecutive k -> one 16-byte read, for A (rows = m) and B (rows = n).
        const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < T::NKK; ++kk) {
            const int ra_ = wm * T::WM + l32, rb_ = wn * T::WN + l32;
            a_frag[kk] = ra_ * T::ROW + T::swz(ra_, kk * 2 + lh) * 16;
            b_frag[kk] = T::A_STAGE + rb_ * T::ROW + T::swz(rb_, kk * 2 + lh) * 16;
        }
        // Output: accumulator register v of MFMA tile (mi, ni) is row 8*(v/4) + 4*(lane/32) + v%4,
        // column lane%32 of that 32x32 tile.
        c_voff = (uint32_t)(wm * T::WM + 4 * lh) * p.ldc_b + (uint32_t)(wn * T::WN + l32) * T::ES;
        c_colb = (uint32_t)z * T::TN * T::ES + (uint32_t)(wn * T::WN + l32) * T::ES;
    }

    // Ragged K.  True (uniformly) in the y steps in which the last block column of A reaches past K.
    LCMA_DEV bool k_tail(int y) const { return (uint32_t)(y + 1) * (T::TK * T::ES) > p.k_tail_b; }
    // In such a step: `voff` if the 16-byte chunk at byte column `colb` of the matrix lies inside K,
    // else the end of the extent (the load returns zero).  The column of a thread's chunk is worked
    // out again from its thread index there rather than kept in a register through the whole loop.
    LCMA_DEV uint32_t a_inside(uint32_t voff, uint32_t colb) const { return colb < p.k_row_b ? voff : p.a_bytes; }
    // `guard` is a literal at every call site: the steps before the tail carry no guard code at all.
    LCMA_DEV u32x4 load_a(int q, uint32_t soff, int l, int y, bool guard) const {
        uint32_t vo = a_voff[q];
        if (guard) {
            const int c = ((q * T::NT + (int)threadIdx.x) % T::NCHK_A) % T::CPR;
            vo = a_inside(vo, (uint32_t)l * p.a_bcol + (uint32_t)y * (T::TK * T::ES) + c * 16);
        }
        return __builtin_amdgcn_raw_buffer_load_b128(ra, (int)vo, (int)soff, 0);
    }
    // Offset of B unit q in block column j: past N the lane reads from the end of the extent (zero).
    // (c_bcol is the width of a block of B and C in bytes of n, whichever way B is stored.)
    LCMA_DEV uint32_t b_voff_in(int q, int j) const {
        return ((uint32_t)j * p.c_bcol + b_colb[q] < p.n_row_b) ? b_voff[q] : p.b_bytes;
    }
    // B given N x K: chunk q of the tile of B_{l,j}; what lies past K must read as zero here too,
    // because a row of W continues with padding or with the next row.
    LCMA_DEV u32x4 load_bt(int q, uint32_t soff, int l, int j, int y, bool guard) const {
        uint32_t vo = b_voff_in(q, j);
        if (guard) {
            const int c = ((q * T::NT + (int)threadIdx.x) % T::NU_B) % T::CPR;
            if ((uint32_t)l * p.b_brow + (uint32_t)y * (T::TK * T::ES) + c * 16 >= p.k_row_b) vo = p.b_bytes;
        }
        return __builtin_amdgcn_raw_buffer_load_b128(rb, (int)vo, (int)soff, 0);
    }
    LCMA_DEV uint32_t load_b(uint32_t voff, uint32_t soff) const {
        return __builtin_amdgcn_raw_buffer_load_b32(rb, (int)voff, (int)soff, 0);
    }
    // Scalar byte offset of tile y of block A_{i,l} / B_{l,j} for this group.
    LCMA_DEV uint32_t soff_a(int i, int l, int y) const {
        return (uint32_t)i * p.a_brow + (uint32_t)l * p.a_bcol + a_group + (uint32_t)y * (T::TK * T::ES);
    }
    LCMA_DEV uint32_t soff_b(int l, int j, int y) const {
        return (uint32_t)l * p.b_brow + (uint32_t)j * p.b_bcol + b_group +
               (T::TB ? (uint32_t)y * (T::TK * T::ES) : (uint32_t)y * T::TK * p.ldb_b);
    }

    LCMA_DEV void lds_store(uint32_t off, const u32x4 &v) const { *(LCMA_LDS u32x4 *)(lds + off) = v; }
    LCMA_DEV Frag lds_frag(uint32_t off) const { return __builtin_bit_cast(Frag, *(LCMA_LDS u32x4 *)(lds + off)); }

    // acc[s] += At_s x Bt_s for the NP products whose combinations sit in LDS stage `st`.
    template <int NP> LCMA_DEV void mma_stage(int st, typename T::Acc (&acc)[NP]) const {
        const uint32_t sb = st * T::STAGE;
#pragma unroll
        for (int s = 0; s < NP; ++s) {
#pragma unroll
            for (int kk = 0; kk < T::NKK; ++kk) {
                Frag a[T::NMI], b[T::NNI];
#pragma unroll
                for (int mi = 0; mi < T::NMI; ++mi) a[mi] = lds_frag(sb + s * T::A_SLOT + a_frag[kk] + mi * 32 * T::ROW);
#pragma unroll
                for (int ni = 0; ni < T::NNI; ++ni) b[ni] = lds_frag(sb + s * T::B_SLOT + b_frag[kk] + ni * 32 * T::ROW);
#pragma unroll
                for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < T::NNI; ++ni) Mma<CT>::run(a[mi], b[ni], acc[s].v[mi][ni]);
            }
        }
    }

    // Fragment-combine form: LDS stage `st` holds the raw blocks; read their fragments once, form the
    // operand fragments of every product with CH::comb_a / comb_b (Eq. 3 / Eq. 4 on registers) and
    // multiply.
    // `hook(slot, slots)` runs after the MFMA instructions of product group `slot` (numbered through
    // all k sub-steps); its instructions issue while those MFMAs execute.
    // Fragments of the raw blocks of one k sub-step, double-buffered.
    template <class CH> struct Frags {
        Frag a[2][T::NMI][CH::NA], b[2][T::NNI][CH::NB];
    };
    template <class CH> LCMA_DEV void fetch_frags(Frags<CH> &f, int st, int kk, int buf) const {
        const uint32_t sb = st * T::STAGE;
#pragma unroll
        for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
            for (int t = 0; t < CH::NA; ++t) f.a[buf][mi][t] = lds_frag(sb + t * T::A_SLOT + a_frag[kk] + mi * 32 * T::ROW);
#pragma unroll
        for (int ni = 0; ni < T::NNI; ++ni)
#pragma unroll
            for (int t = 0; t < CH::NB; ++t) f.b[buf][ni][t] = lds_frag(sb + t * T::B_SLOT + b_frag[kk] + ni * 32 * T::ROW);
    }
    // The same with the stage given as a pointer: a caller that holds the stage it reads and the stage it
    // fills as two restrict-qualified pointers lets the compiler see that direct loads into the one never
    // alias fragment reads from the other (without that it waits for every direct load in flight before
    // each LDS read that follows one).
    template <class CH> LCMA_DEV void fetch_frags_at(Frags<CH> &f, const LCMA_LDS char *base, int kk, int buf) const {
#pragma unroll
        for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
            for (int t = 0; t < CH::NA; ++t)
                f.a[buf][mi][t] = __builtin_bit_cast(Frag, *(const LCMA_LDS u32x4 *)(base + t * T::A_SLOT + a_frag[kk] + mi * 32 * T::ROW));
#pragma unroll
        for (int ni = 0; ni < T::NNI; ++ni)
#pragma unroll
            for (int t = 0; t < CH::NB; ++t)
                f.b[buf][ni][t] = __builtin_bit_cast(Frag, *(const LCMA_LDS u32x4 *)(base + t * T::B_SLOT + b_frag[kk] + ni * 32 * T::ROW));
    }
    template <class CH, class HOOK>
    LCMA_DEV void mma_stage_fc_at(const LCMA_LDS char *base, typename T::Acc (&acc)[CH::NP], HOOK hook) const {
        Frags<CH> f;
        fetch_frags_at<CH>(f, base, 0, 0);
#pragma unroll
        for (int kk = 0; kk < T::NKK; ++kk) {
            const int cur = kk & 1;
            if (kk + 1 < T::NKK) fetch_frags_at<CH>(f, base, kk + 1, cur ^ 1);
            combine_and_multiply<CH>(f, cur, kk, acc, hook);
        }
    }
    template <class CH> LCMA_DEV void mma_stage_fc(int st, typename T::Acc (&acc)[CH::NP]) const {
        mma_stage_fc<CH>(st, acc, [](int, int) {});
    }
    template <class CH, class HOOK>
    LCMA_DEV void mma_stage_fc(int st, typename T::Acc (&acc)[CH::NP], HOOK hook) const {
        Frags<CH> f;
        fetch_frags<CH>(f, st, 0, 0);
        mma_stage_fc<CH>(st, -1, f, acc, hook);
    }
    // `f` holds the fragments of k sub-step 0 of stage `st` in buffer 0 on entry.  With nst >= 0 the
    // fragments of k sub-step 0 of stage `nst` are fetched into buffer 0 under the last sub-step's
    // MFMAs (needs an even number of sub-steps).  `hook(slot, slots)` runs after the MFMA instructions
    // of product group `slot` (numbered through all k sub-steps); its instructions issue while those
    // MFMAs execute.
    template <class CH, class HOOK>
    LCMA_DEV void mma_stage_fc(int st, int nst, Frags<CH> &f, typename T::Acc (&acc)[CH::NP], HOOK hook) const {
#pragma unroll
        for (int kk = 0; kk < T::NKK; ++kk) {
            const int cur = kk & 1;
            // next fragments arrive under this step's MFMAs
            if (kk + 1 < T::NKK) fetch_frags<CH>(f, st, kk + 1, cur ^ 1);
            else if (nst >= 0) {
                // issued now, a whole k sub-step before the barrier: the barrier waits for every
                // outstanding LDS operation, so reads issued just before it would be waited for there
                fetch_frags<CH>(f, nst, 0, cur ^ 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            combine_and_multiply<CH>(f, cur, kk, acc, hook);
        }
    }

    // One k sub-step of the fragment-combine loop: form the operand fragments of every product from the raw
    // fragments in buffer `cur` and multiply.
    template <class CH, class HOOK>
    LCMA_DEV void combine_and_multiply(Frags<CH> &f, int cur, int kk, typename T::Acc (&acc)[CH::NP], HOOK hook) const {
        // A few products at a time keeps few combined fragments live (the unused outputs of the
        // generated combination code are dead and vanish).  With several MFMA instructions per
        // fragment pair (fp32) two products advance together, so that back-to-back instructions
        // never accumulate into the same tile.
        constexpr int G = (Mma<CT>::SUB > 1 && T::NMI * T::NNI == 1) ? LCMA_FP32_GROUP : 1;
#pragma unroll
        for (int s0 = 0; s0 < CH::NP; s0 += G) {
            Frag at[G][T::NMI], bt[G][T::NNI];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (s0 + g >= CH::NP) continue;
#pragma unroll
                for (int mi = 0; mi < T::NMI; ++mi) {
                    Frag o[CH::NP];
                    CH::comb_a(f.a[cur][mi], o);
                    at[g][mi] = o[s0 + g];
                }
#pragma unroll
                for (int ni = 0; ni < T::NNI; ++ni) {
                    Frag o[CH::NP];
                    CH::comb_b(f.b[cur][ni], o);
                    bt[g][ni] = o[s0 + g];
                }
            }
            mfma_priority(true);
#pragma unroll
            for (int t = 0; t < Mma<CT>::SUB; ++t)
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (s0 + g >= CH::NP) continue;
#pragma unroll
                    for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < T::NNI; ++ni)
                            Mma<CT>::run_sub(at[g][mi], bt[g][ni], acc[s0 + g].v[mi][ni], t);
                }
            mfma_priority(false);
            constexpr int NG = (CH::NP + G - 1) / G;
            hook(kk * NG + s0 / G, T::NKK * NG);
        }
    }

    // Prepared-B form: LDS stage `st` holds the raw A blocks and the tile of Bt_s in B slot s.  The A
    // fragments are read once per k sub-step and combined per product (Eq. 3 on registers); the
    // fragments of Bt_s are used by product s alone, so they stream through two small buffers, each
    // read while the previous product group multiplies.
    template <class CH, class HOOK>
    LCMA_DEV void mma_stage_pb(int st, typename T::Acc (&acc)[CH::NP], HOOK hook) const {
        const uint32_t sb = st * T::STAGE;
        constexpr int G = (Mma<CT>::SUB > 1 && T::NMI * T::NNI == 1) ? LCMA_FP32_GROUP : 1;
        constexpr int NG = (CH::NP + G - 1) / G;
        u32x4 fa[2][T::NMI][CH::NA]; // as they sit in LDS: compute type, or storage type with direct loads
        Frag fb[2][G][T::NNI];
        auto fetch_a = [&](int kk, int buf) {
#pragma unroll
            for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
                for (int t = 0; t < CH::NA; ++t)
                    fa[buf][mi][t] = *(LCMA_LDS u32x4 *)(lds + sb + t * T::A_SLOT + a_frag[kk] + mi * 32 * T::ROW);
        };
        auto fetch_b = [&](int kk, int gi, int buf) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (gi * G + g >= CH::NP) continue;
#pragma unroll
                for (int ni = 0; ni < T::NNI; ++ni)
                    fb[buf][g][ni] = lds_frag(sb + (gi * G + g) * T::B_SLOT + b_frag[kk] + ni * 32 * T::ROW);
            }
        };
        fetch_a(0, 0);
        fetch_b(0, 0, 0);
#pragma unroll
        for (int kk = 0; kk < T::NKK; ++kk) {
            const int cur = kk & 1;
            if (kk + 1 < T::NKK) fetch_a(kk + 1, cur ^ 1);
            Frag ca[T::NMI][CH::NA];
#pragma unroll
            for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
                for (int t = 0; t < CH::NA; ++t) {
                    if constexpr (T::DL) ca[mi][t] = __builtin_bit_cast(Frag, Convert<IN, CT>::run(fa[cur][mi][t]));
                    else ca[mi][t] = __builtin_bit_cast(Frag, fa[cur][mi][t]);
                }
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                const int flat = kk * NG + gi, bcur = flat & 1;
                if (gi + 1 < NG) fetch_b(kk, gi + 1, bcur ^ 1);
                else if (kk + 1 < T::NKK) fetch_b(kk + 1, 0, bcur ^ 1);
                Frag at[G][T::NMI];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (gi * G + g >= CH::NP) continue;
#pragma unroll
                    for (int mi = 0; mi < T::NMI; ++mi) {
                        Frag o[CH::NP];
                        CH::comb_a(ca[mi], o);
                        at[g][mi] = o[gi * G + g];
                    }
                }
#pragma unroll
                for (int t = 0; t < Mma<CT>::SUB; ++t)
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        if (gi * G + g >= CH::NP) continue;
#pragma unroll
                        for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
                            for (int ni = 0; ni < T::NNI; ++ni)
                                Mma<CT>::run_sub(at[g][mi], fb[bcur][g][ni], acc[gi * G + g].v[mi][ni], t);
                    }
                hook(flat, T::NKK * NG);
            }
        }
    }

    // alpha * acc + beta * (the element of C at byte offset off + soff), in fp32.  C is read only when beta is
    // not zero (uniform over the launch), with one small load per element in the accumulator layout: the general
    // scaling is a convenience, not a fast path.
    LCMA_DEV float scaled(float acc, uint32_t off, uint32_t soff) const {
        float o = p.alpha * acc;
        if (p.beta != 0.f) {
            float old;
            if constexpr (T::ES == 2) {
                const uint32_t bits = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rc, (int)off, (int)soff, 0);
                if constexpr (std::is_same_v<IN, BF16>) old = __builtin_bit_cast(float, bits << 16);
                else old = (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
            } else {
                old = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rc, (int)off, (int)soff, 0));
            }
            o = __builtin_fmaf(p.beta, old, o);
        }
        return o;
    }
    // Byte offset (without soff) of accumulator value v of MFMA tile (mi, ni) of this lane; past N: the end of the extent.
    LCMA_DEV uint32_t elem_off(int j, int mi, int ni, int v) const {
        const uint32_t base = ((uint32_t)j * p.c_bcol + c_colb + ni * 32 * T::ES < p.n_row_b) ? c_voff : p.c_bytes;
        return base + (uint32_t)(mi * 32 + (v >> 2) * 8 + (v & 3)) * p.ldc_b + ni * 32 * T::ES;
    }

    // Round and store one fp32 tile into block C_{i,j}.  f(mi, ni) returns the f32x16 of MFMA
    // tile (mi, ni).
    //
    // 16-bit output: a lane's 16 accumulator values of an MFMA tile lie in ONE column, so storing them
    // directly takes sixteen 2-byte stores that cover 64 bytes of a row each.  Instead every wave
    // passes one 32-row strip of its tile (32 x WN elements) through a private piece of LDS (the stages
    // are free after the y loop) and writes it out with 16-byte stores, whole 128-byte lines when the
    // wave tile is 64 columns wide: 8x fewer store instructions.  All waves of the work-group call this
    // together; the barriers keep the strip apart from the stage buffers of the loop before and after.
    template <class F> LCMA_DEV void store_c(int i, int j, F f) const {
        const uint32_t soff = (uint32_t)i * p.c_brow + (uint32_t)j * p.c_bcol + c_group;
        if constexpr (T::ES == 2 && LCMA_EPILOGUE_LDS) {
            constexpr int PITCH = T::WN * 2 + 16;          // bytes; rows 4 apart fall into different banks
            constexpr int CPRW = T::WN * 2 / 16;           // 16-byte chunks per strip row
            constexpr int NIT = 32 * CPRW / 64;            // chunks per lane
            static_assert(T::NT / 64 * 32 * PITCH <= T::LDS_BYTES, "the strips of all waves fit the stage buffers");
            LCMA_LDS char *strip = lds + (threadIdx.x >> 6) * (32 * PITCH);
            const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
            for (int mi = 0; mi < T::NMI; ++mi) {
#pragma unroll
                for (int ni = 0; ni < T::NNI; ++ni) {
                    const f32x16 t = f(mi, ni);
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        *(LCMA_LDS uint16_t *)(strip + ((v >> 2) * 8 + 4 * lh + (v & 3)) * PITCH + (ni * 32 + l32) * 2) =
                            (uint16_t)Round<IN>::run(scaled(t[v], elem_off(j, mi, ni, v), soff));
                }
                __syncthreads();
#pragma unroll
                for (int it = 0; it < NIT; ++it) {
                    const int id = it * 64 + lane, row = id / CPRW, ch = id % CPRW;
                    const u32x4 v = *(LCMA_LDS u32x4 *)(strip + row * PITCH + ch * 16);
                    const uint32_t colb = (uint32_t)(wn * T::WN) * 2 + ch * 16; // byte column inside the tile
                    // a chunk past N goes to the end of the extent: dropped (N is a whole number of chunks)
                    const uint32_t off = ((uint32_t)j * p.c_bcol + n_group + colb < p.n_row_b)
                                             ? (uint32_t)(wm * T::WM + mi * 32 + row) * p.ldc_b + colb
                                             : p.c_bytes;
                    // The scalar offset is added to the vector offset and the scalar-offset field left a
                    // literal zero on purpose.  A store of more than 8 bytes reads its data registers over
                    // several cycles; the compiler keeps a following vector write to those registers at a
                    // distance only when the store has no scalar-register offset.  With one, on MI355X, the
                    // next row's address computation (which had been given the first data register)
                    // overwrote the data of the last quarter of the lanes.
                    __builtin_amdgcn_raw_buffer_store_b128(v, rc, (int)(off + soff), 0, 0);
                }
                __syncthreads();
            }
        } else {
#pragma unroll
        for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
            for (int ni = 0; ni < T::NNI; ++ni) {
                const f32x16 t = f(mi, ni);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // a lane whose column lies past N stores to the end of the extent: dropped
                    const uint32_t off = elem_off(j, mi, ni, v);
                    const uint32_t bits = Round<IN>::run(scaled(t[v], off, soff));
                    if constexpr (T::ES == 2)
                        __builtin_amdgcn_raw_buffer_store_b16((short)bits, rc, (int)off, (int)soff, 0);
                    else
                        __builtin_amdgcn_raw_buffer_store_b32(bits, rc, (int)off, (int)soff, 0);
                }
            }
        }
    }
};

// ---------------------------------------------------------------- one chunk of products over all y
// CH (generated) describes the chunk:
//   NA, NB, NP        raw A blocks, raw B blocks, products
//   a_i(t), a_l(t)    block indices of raw A block t; b_l(t), b_j(t) likewise for B
//   comb_a(in, out)   out[s] = sum_t U * in[t]  (Eq. 3) on 16-byte vectors; comb_b likewise (Eq. 4)
template <class T, class CH> struct RawSet {
    u32x4 a[T::PA ? CH::NP : CH::NA][T::QA]; // raw blocks, or with ready-made left operands one tile of At_r per product
    // B side: raw blocks (units of BH vectors), or with prepared B one tile of Bt_r per product
    u32x4 b[T::PB ? CH::NP : CH::NB][T::PB ? T::QBP : T::QB][T::PB ? 1 : T::BH];
};

// Issue the buffer loads of step y into `r`.
template <class T, class CH> LCMA_DEV void issue_loads(const Ctx<T> &cx, RawSet<T, CH> &r, int y, bool guard) {
    if constexpr (T::PA) { // planes are padded with zeros: nothing to guard
#pragma unroll
        for (int s = 0; s < CH::NP; ++s) {
            const uint32_t so = (uint32_t)CH::a_plane(s) * cx.p.a_brow + cx.a_group + (uint32_t)y * (T::TK * T::ES);
#pragma unroll
            for (int q = 0; q < T::QA; ++q)
                r.a[s][q] = __builtin_amdgcn_raw_buffer_load_b128(cx.ra, (int)cx.a_voff[q], (int)so, 0);
        }
    } else {
#pragma unroll
        for (int t = 0; t < CH::NA; ++t) {
            const uint32_t so = cx.soff_a(CH::a_i(t), CH::a_l(t), y);
#pragma unroll
            for (int q = 0; q < T::QA; ++q) r.a[t][q] = cx.load_a(q, so, CH::a_l(t), y, guard);
        }
    }
    if constexpr (T::PB) {
#pragma unroll
        for (int s = 0; s < CH::NP; ++s) {
            const uint32_t so = (uint32_t)CH::b_plane(s) * cx.p.b_brow + cx.b_group + (uint32_t)y * (T::TK * T::ES);
#pragma unroll
            for (int q = 0; q < T::QBP; ++q)
                r.b[s][q][0] = __builtin_amdgcn_raw_buffer_load_b128(cx.rb, (int)cx.bp_voff[q], (int)so, 0);
        }
    } else {
#pragma unroll
        for (int t = 0; t < CH::NB; ++t) {
            const uint32_t so = cx.soff_b(CH::b_l(t), CH::b_j(t), y);
#pragma unroll
            for (int q = 0; q < T::QB; ++q) {
                if constexpr (T::TB) {
                    r.b[t][q][0] = cx.load_bt(q, so, CH::b_l(t), CH::b_j(t), y, guard);
                } else {
                    const uint32_t vo = cx.b_voff_in(q, CH::b_j(t));
#pragma unroll
                    for (int e = 0; e < T::BW; ++e) r.b[t][q][e / 4][e % 4] = cx.load_b(vo, so + (uint32_t)e * cx.p.ldb_b);
                }
            }
        }
    }
}

// Convert the raw blocks in `r`, form the combinations (Eq. 3 / Eq. 4) unless the kernel combines
// fragments later, transpose B to k-contiguous chunks and write everything to LDS stage `st`.
template <class T, class CH> LCMA_DEV void combine_store(const Ctx<T> &cx, const RawSet<T, CH> &r, int st) {
    using V = typename T::CT::vec;
    using Cv = Convert<typename T::IN, typename T::CT>;
    constexpr int NOA = T::FC ? CH::NA : CH::NP, NOB = T::FC ? CH::NB : CH::NP;
    static_assert(NOA <= T::NSA && NOB <= T::NSB, "chunk larger than the LDS slots");
    const uint32_t sb = st * T::STAGE;
    if constexpr (T::PA) { // tiles of At_r go to LDS as they are
#pragma unroll
        for (int s = 0; s < CH::NP; ++s)
#pragma unroll
            for (int q = 0; q < T::QA; ++q) cx.lds_store(sb + s * T::A_SLOT + cx.a_lds[q], r.a[s][q]);
    } else {
#pragma unroll
    for (int q = 0; q < T::QA; ++q) {
        V in[CH::NA], out[NOA];
#pragma unroll
        for (int t = 0; t < CH::NA; ++t) in[t] = Cv::run(r.a[t][q]);
        if constexpr (T::FC) {
#pragma unroll
            for (int t = 0; t < CH::NA; ++t) out[t] = in[t];
        } else {
            CH::comb_a(in, out);
        }
#pragma unroll
        for (int s = 0; s < NOA; ++s) cx.lds_store(sb + s * T::A_SLOT + cx.a_lds[q], __builtin_bit_cast(u32x4, out[s]));
    }
    }
    if constexpr (T::PB) { // tiles of Bt_r go to LDS as they are
#pragma unroll
        for (int s = 0; s < CH::NP; ++s)
#pragma unroll
            for (int q = 0; q < T::QBP; ++q) cx.lds_store(sb + s * T::B_SLOT + cx.bp_lds[q], r.b[s][q][0]);
        return;
    } else {
#pragma unroll
    for (int q = 0; q < T::QB; ++q) {
        V out[T::BH][NOB];
#pragma unroll
        for (int h = 0; h < T::BH; ++h) {
            V in[CH::NB];
#pragma unroll
            for (int t = 0; t < CH::NB; ++t) in[t] = Cv::run(r.b[t][q][h]);
            if constexpr (T::FC) {
#pragma unroll
                for (int t = 0; t < CH::NB; ++t) out[h][t] = in[t];
            } else {
                CH::comb_b(in, out[h]);
            }
        }
#pragma unroll
        for (int s = 0; s < NOB; ++s) {
            if constexpr (T::TB) { // a chunk of a row n: k-contiguous already
                cx.lds_store(sb + s * T::B_SLOT + cx.b_lds[q], __builtin_bit_cast(u32x4, out[0][s]));
            } else if constexpr (T::ES == 2) {
                // dword e of the unit holds columns (2c, 2c+1) at k = k0 + e; gather the low halves
                // into the chunk of column 2c and the high halves into the chunk of column 2c+1
                const u32x4 lo = __builtin_bit_cast(u32x4, out[0][s]), hi = __builtin_bit_cast(u32x4, out[1][s]);
                u32x4 c0, c1;
                c0[0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x05040100u);
                c0[1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x05040100u);
                c0[2] = __builtin_amdgcn_perm(hi[1], hi[0], 0x05040100u);
                c0[3] = __builtin_amdgcn_perm(hi[3], hi[2], 0x05040100u);
                c1[0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u);
                c1[1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u);
                c1[2] = __builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u);
                c1[3] = __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u);
                cx.lds_store(sb + s * T::B_SLOT + cx.b_lds[q], c0);
                cx.lds_store(sb + s * T::B_SLOT + cx.b_lds1[q], c1);
            } else {
                cx.lds_store(sb + s * T::B_SLOT + cx.b_lds[q], __builtin_bit_cast(u32x4, out[0][s]));
            }
        }
    }
    }
}

// Fragment-combine kernels stage the raw blocks only, so which block a thread stages need not be the
// same for every thread: all chunks (A) and units (B) of all blocks form one pool that is dealt to
// the threads, which avoids idle or duplicated staging work when a single block is small.
template <class T, class CH> struct FlatStage {
    static constexpr int NCHK_B = T::TN * T::CPR; // 16-byte chunks of one prepared-B tile
    static constexpr int NCA = CH::NA * T::NCHK_A, NUB = T::PB ? CH::NP * NCHK_B : CH::NB * T::NU_B;
    static constexpr int QA = (NCA + T::NT - 1) / T::NT, QB = (NUB + T::NT - 1) / T::NT;
    uint32_t a_voff[QA], a_lds[QA], b_voff[QB], b_lds[QB], b_lds1[QB];
    struct Raw {
        u32x4 a[QA], b[QB][T::PB ? 1 : T::BH];
    };

    LCMA_DEV FlatStage(const Ctx<T> &cx) {
        const int tid = threadIdx.x;
#pragma unroll
        for (int q = 0; q < QA; ++q) {
            const int id = (q * T::NT + tid) % NCA;
            const int t = id / T::NCHK_A, id2 = id % T::NCHK_A;
            const int row = id2 / T::CPR, c = id2 % T::CPR;
            a_voff[q] = (uint32_t)CH::a_i(t) * cx.p.a_brow + (uint32_t)CH::a_l(t) * cx.p.a_bcol +
                        (uint32_t)row * cx.p.lda_b + c * 16;
            a_lds[q] = t * T::A_SLOT + row * T::ROW + T::swz(row, c) * 16;
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int id = (q * T::NT + tid) % NUB;
            if constexpr (T::PB) {
                // plane s of the prepared operand: rows n of this group's tile, k-contiguous
                const int sl = id / NCHK_B, id2 = id % NCHK_B;
                const int row = id2 / T::CPR, c = id2 % T::CPR;
                b_voff[q] = (uint32_t)sl * cx.p.b_brow + (uint32_t)row * cx.p.ldb_b + c * 16;
                b_lds[q] = T::A_STAGE + sl * T::B_SLOT + row * T::ROW + T::swz(row, c) * 16;
                b_lds1[q] = 0;
            } else if constexpr (T::TB) {
                // B given N x K: chunk c of row n of block B_{l,j}, handled like a chunk of A
                const int t = id / T::NU_B, u = id % T::NU_B;
                const int row = u / T::CPR, c = u % T::CPR;
                b_voff[q] = (uint32_t)CH::b_l(t) * cx.p.b_brow + (uint32_t)CH::b_j(t) * cx.p.b_bcol +
                            (uint32_t)row * cx.p.ldb_b + c * 16;
                // rows past N: read from the end of the extent (zero) for the whole run
                const uint32_t n_b = cx.n_group + (uint32_t)row * T::ES; // n inside the block, in bytes of a row of C
                if ((uint32_t)CH::b_j(t) * cx.p.c_bcol + n_b >= cx.p.n_row_b) b_voff[q] = cx.p.b_bytes;
                b_lds[q] = T::A_STAGE + t * T::B_SLOT + row * T::ROW + T::swz(row, c) * 16;
                b_lds1[q] = 0;
            } else {
                const int t = id / T::NU_B, u = id % T::NU_B;
                const int col = u % T::BCOLS, g = u / T::BCOLS;
                const int row = (T::ES == 2) ? 2 * col : col;
                b_voff[q] = (uint32_t)CH::b_l(t) * cx.p.b_brow + (uint32_t)CH::b_j(t) * cx.p.b_bcol +
                            (uint32_t)(g * T::CH) * cx.p.ldb_b + col * 4;
                // columns past N: read from the end of the extent (zero) for the whole run
                if ((uint32_t)CH::b_j(t) * cx.p.b_bcol + cx.b_group + col * 4 >= cx.p.n_row_b) b_voff[q] = cx.p.b_bytes;
                b_lds[q] = T::A_STAGE + t * T::B_SLOT + row * T::ROW + T::swz(row, g) * 16;
                b_lds1[q] = T::A_STAGE + t * T::B_SLOT + (row + 1) * T::ROW + T::swz(row + 1, g) * 16;
            }
        }
    }
    // offset of A chunk q in step y (ragged K: the end of the extent when the chunk lies past K)
    LCMA_DEV uint32_t a_off(const Ctx<T> &cx, int q, int y, bool guard) const {
        uint32_t vo = a_voff[q];
        if (guard) {
            const int id = (q * T::NT + (int)threadIdx.x) % NCA;
            const int t = id / T::NCHK_A, c = (id % T::NCHK_A) % T::CPR;
            vo = cx.a_inside(vo, (uint32_t)CH::a_l(t) * cx.p.a_bcol + (uint32_t)y * (T::TK * T::ES) + c * 16);
        }
        return vo;
    }
    LCMA_DEV void load_b(const Ctx<T> &cx, Raw &r, int q, int y, bool guard) const {
        if constexpr (T::PB) {
            const uint32_t sbo = cx.b_group + (uint32_t)y * (T::TK * T::ES);
            r.b[q][0] = __builtin_amdgcn_raw_buffer_load_b128(cx.rb, (int)b_voff[q], (int)sbo, 0);
        } else if constexpr (T::TB) {
            const uint32_t sbo = cx.b_group + (uint32_t)y * (T::TK * T::ES);
            uint32_t vo = b_voff[q];
            if (guard) { // past K a row of W goes on with padding or the next row: read zero instead
                const int id = (q * T::NT + (int)threadIdx.x) % NUB;
                const int t = id / T::NU_B, c = (id % T::NU_B) % T::CPR;
                if ((uint32_t)CH::b_l(t) * cx.p.b_brow + (uint32_t)y * (T::TK * T::ES) + c * 16 >= cx.p.k_row_b) vo = cx.p.b_bytes;
            }
            r.b[q][0] = __builtin_amdgcn_raw_buffer_load_b128(cx.rb, (int)vo, (int)sbo, 0);
        } else {
            const uint32_t sbo = cx.b_group + (uint32_t)y * T::TK * cx.p.ldb_b;
#pragma unroll
            for (int e = 0; e < T::BW; ++e)
                r.b[q][e / 4][e % 4] = __builtin_amdgcn_raw_buffer_load_b32(
                    cx.rb, (int)b_voff[q], (int)(sbo + (uint32_t)e * cx.p.ldb_b), 0);
        }
    }
    LCMA_DEV void issue(const Ctx<T> &cx, Raw &r, int y, bool guard) const {
        const uint32_t sa = cx.a_group + (uint32_t)y * (T::TK * T::ES);
#pragma unroll
        for (int q = 0; q < QA; ++q) r.a[q] = __builtin_amdgcn_raw_buffer_load_b128(cx.ra, (int)a_off(cx, q, y, guard), (int)sa, 0);
#pragma unroll
        for (int q = 0; q < QB; ++q) load_b(cx, r, q, y, guard);
    }
    // The staging work of one thread cut into NPIECE pieces (one 16-byte A chunk or one B unit each),
    // so that it can be spread over the MFMA phase.
    static constexpr int NPIECE = QA + QB;
    LCMA_DEV void issue_piece(const Ctx<T> &cx, Raw &r, int pc, int y, bool guard) const {
        if (pc < QA) {
            const uint32_t sa = cx.a_group + (uint32_t)y * (T::TK * T::ES);
            r.a[pc] = __builtin_amdgcn_raw_buffer_load_b128(cx.ra, (int)a_off(cx, pc, y, guard), (int)sa, 0);
        } else {
            load_b(cx, r, pc - QA, y, guard);
        }
    }
    LCMA_DEV void store_piece(const Ctx<T> &cx, const Raw &r, int pc, int st) const {
        const uint32_t sb = st * T::STAGE;
        if (pc < QA) store_a(cx, r, pc, sb);
        else store_b(cx, r, pc - QA, sb);
    }
    LCMA_DEV void store(const Ctx<T> &cx, const Raw &r, int st) const {
        const uint32_t sb = st * T::STAGE;
#pragma unroll
        for (int q = 0; q < QA; ++q) store_a(cx, r, q, sb);
#pragma unroll
        for (int q = 0; q < QB; ++q) store_b(cx, r, q, sb);
    }
    LCMA_DEV void store_a(const Ctx<T> &cx, const Raw &r, int q, uint32_t sb) const {
        using Cv = Convert<typename T::IN, typename T::CT>;
        cx.lds_store(sb + a_lds[q], __builtin_bit_cast(u32x4, Cv::run(r.a[q])));
    }
    LCMA_DEV void store_b(const Ctx<T> &cx, const Raw &r, int q, uint32_t sb) const {
        using Cv = Convert<typename T::IN, typename T::CT>;
        if constexpr (T::PB) {
            cx.lds_store(sb + b_lds[q], r.b[q][0]); // already in the compute type and k-contiguous
        } else if constexpr (T::TB) {
            cx.lds_store(sb + b_lds[q], __builtin_bit_cast(u32x4, Cv::run(r.b[q][0]))); // k-contiguous already
        } else {
            if constexpr (T::ES == 2) {
                const u32x4 lo = __builtin_bit_cast(u32x4, Cv::run(r.b[q][0]));
                const u32x4 hi = __builtin_bit_cast(u32x4, Cv::run(r.b[q][1]));
                u32x4 c0, c1;
                c0[0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x05040100u);
                c0[1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x05040100u);
                c0[2] = __builtin_amdgcn_perm(hi[1], hi[0], 0x05040100u);
                c0[3] = __builtin_amdgcn_perm(hi[3], hi[2], 0x05040100u);
                c1[0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u);
                c1[1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u);
                c1[2] = __builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u);
                c1[3] = __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u);
                cx.lds_store(sb + b_lds[q], c0);
                cx.lds_store(sb + b_lds1[q], c1);
            } else {
                cx.lds_store(sb + b_lds[q], __builtin_bit_cast(u32x4, Cv::run(r.b[q][0])));
            }
        }
    }
};

// Direct loads: the LDS image of a stage is linear in 16-byte chunks, a wave instruction fills 64
// consecutive chunks (lane l lands at base + 16 l), and the swizzle is applied by choosing which
// chunk of memory each lane fetches.  Pieces are whole work-group instructions; in the last piece of
// a side the waves past the end skip (wave-uniform).
template <class T, class CH> struct DirectStage {
    static constexpr int NCHK_B = T::TN * T::CPR;
    static constexpr int NCA = CH::NA * T::NCHK_A, NCB = (T::PB ? CH::NP : CH::NB) * NCHK_B;
    static_assert(NCA % 64 == 0 && NCB % 64 == 0, "a wave instruction must not straddle the end of a side");
    static constexpr int QA = (NCA + T::NT - 1) / T::NT, QB = (NCB + T::NT - 1) / T::NT;
    static constexpr int NPIECE = QA + QB;
    uint32_t a_voff[QA], b_voff[QB];
    int wave_chunk; // first chunk of this wave inside a piece (wave-uniform)

    LCMA_DEV DirectStage(const Ctx<T> &cx) {
        const int tid = threadIdx.x;
        wave_chunk = __builtin_amdgcn_readfirstlane(tid & ~63);
#pragma unroll
        for (int q = 0; q < QA; ++q) {
            const int pp = (q * T::NT + tid) % NCA;
            const int t = pp / T::NCHK_A, id2 = pp % T::NCHK_A;
            const int row = id2 / T::CPR, cs = id2 % T::CPR;
            // LDS position cs of the row holds memory chunk swz(row, cs) (the XOR is its own inverse)
            a_voff[q] = (uint32_t)CH::a_i(t) * cx.p.a_brow + (uint32_t)CH::a_l(t) * cx.p.a_bcol +
                        (uint32_t)row * cx.p.lda_b + T::swz(row, cs) * 16;
        }
#pragma unroll
        for (int q = 0; q < QB; ++q) {
            const int pp = (q * T::NT + tid) % NCB;
            const int sl = pp / NCHK_B, id2 = pp % NCHK_B;
            const int row = id2 / T::CPR, cs = id2 % T::CPR;
            if constexpr (T::PB) {
                b_voff[q] = (uint32_t)sl * cx.p.b_brow + (uint32_t)row * cx.p.ldb_b + T::swz(row, cs) * 16;
            } else { // raw block sl of B given N x K; rows past N read from the end of the extent (zero)
                b_voff[q] = (uint32_t)CH::b_l(sl) * cx.p.b_brow + (uint32_t)CH::b_j(sl) * cx.p.b_bcol +
                            (uint32_t)row * cx.p.ldb_b + T::swz(row, cs) * 16;
                if ((uint32_t)CH::b_j(sl) * cx.p.c_bcol + cx.n_group + (uint32_t)row * T::ES >= cx.p.n_row_b)
                    b_voff[q] = cx.p.b_bytes;
            }
        }
    }
    LCMA_DEV void issue_piece(const Ctx<T> &cx, int pc, int st, int y, bool guard) const {
        issue_piece_at(cx, pc, cx.lds + st * T::STAGE, y, guard);
    }
    // `stage`: first byte of the LDS stage to fill
    LCMA_DEV void issue_piece_at(const Ctx<T> &cx, int pc, LCMA_LDS char *stage, int y, bool guard) const {
        if (pc < QA) {
            const int first = pc * T::NT + wave_chunk;
            uint32_t vo = a_voff[pc];
            if (guard) {
                const int pp = (pc * T::NT + (int)threadIdx.x) % NCA;
                const int t = pp / T::NCHK_A, row = (pp % T::NCHK_A) / T::CPR, cs = (pp % T::NCHK_A) % T::CPR;
                vo = cx.a_inside(vo, (uint32_t)CH::a_l(t) * cx.p.a_bcol + (uint32_t)y * (T::TK * T::ES) + T::swz(row, cs) * 16);
            }
            if (first < NCA)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(cx.ra, (LCMA_LDS void *)(stage + first * 16), 16,
                                                         (int)vo, (int)(cx.a_group + (uint32_t)y * (T::TK * T::ES)), 0, 0);
        } else {
            const int q = pc - QA, first = q * T::NT + wave_chunk;
            uint32_t vo = b_voff[q];
            if constexpr (!T::PB) {
                if (guard) { // past K a row of W goes on with padding or the next row
                    const int pp = (q * T::NT + (int)threadIdx.x) % NCB;
                    const int t = pp / NCHK_B, row = (pp % NCHK_B) / T::CPR, cs = (pp % NCHK_B) % T::CPR;
                    if ((uint32_t)CH::b_l(t) * cx.p.b_brow + (uint32_t)y * (T::TK * T::ES) + T::swz(row, cs) * 16 >= cx.p.k_row_b)
                        vo = cx.p.b_bytes;
                }
            }
            if (first < NCB)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    cx.rb, (LCMA_LDS void *)(stage + T::A_STAGE + first * 16), 16, (int)vo,
                    (int)(cx.b_group + (uint32_t)y * (T::TK * T::ES)), 0, 0);
        }
    }
    LCMA_DEV void issue(const Ctx<T> &cx, int st, int y) const {
#pragma unroll
        for (int pc = 0; pc < NPIECE; ++pc) issue_piece(cx, pc, st, y, true);
    }
    // every direct load of this wave has landed in LDS
    static LCMA_DEV void landed() { __builtin_amdgcn_s_waitcnt(0x0F70); } // vmcnt(0)
    // Work-group barrier that leaves the NEWEST direct loads of every wave in flight: each wave waits until all
    // but its newest NEWEST loads have landed and its own LDS operations are done (vmcnt(NEWEST) lgkmcnt(0)), then
    // the waves meet.  __syncthreads() cannot be used here: its fences order the LDS writes of the loads in flight
    // as well, so the compiler makes every wave wait for all of them.  The empty asm statements keep the
    // compiler from moving LDS accesses across the bare barrier instruction.
    template <int NEWEST> static LCMA_DEV void barrier_keeping() {
        static_assert(NEWEST >= 0 && NEWEST < 64, "vmcnt has six bits");
        __builtin_amdgcn_s_waitcnt((NEWEST & 0xF) | 0x0070 | ((NEWEST >> 4) << 14));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
};

// One step of the direct-load loop: multiply out of the stage at `rd` while the tiles of step `nxt` travel
// into the stage at `wr`, one work-group load instruction after each product group.  The two stages come in
// as restrict-qualified pointers: that is what tells the compiler that the loads in flight do not touch what
// the fragment reads read, so that it does not wait for them before every LDS read.
template <class T, class CH, bool GUARD>
LCMA_DEV void direct_load_step(const Ctx<T> &cx, const DirectStage<T, CH> &dl, const LCMA_LDS char *__restrict__ rd,
                               LCMA_LDS char *__restrict__ wr, int nxt, typename T::Acc (&acc)[CH::NP]) {
    using DS = DirectStage<T, CH>;
    cx.template mma_stage_fc_at<CH>(rd, acc, [&](int slot, int slots) {
#pragma unroll
        for (int pc = 0; pc < DS::NPIECE; ++pc)
            if (pc * slots / DS::NPIECE == slot) {
                __builtin_amdgcn_sched_barrier(0);
                dl.issue_piece_at(cx, pc, wr, nxt, GUARD);
                __builtin_amdgcn_sched_barrier(0);
            }
    });
}

template <class T, class CH> LCMA_DEV void mma_step(const Ctx<T> &cx, int st, typename T::Acc (&acc)[CH::NP]) {
    if constexpr (T::FC) cx.template mma_stage_fc<CH>(st, acc);
    else cx.template mma_stage<CH::NP>(st, acc);
}

// Runs step(y, y & 1) for y = 0 .. ny-1.  With LIT the loop is unrolled twice so that the stage is a
// literal at both call sites and every LDS address becomes a register plus an immediate.  The address
// arithmetic this saves is worth 5-10% in the 16-bit kernels (bound by vector instruction issue) and
// in the fp32 ones (measured: no cycle in which a VALU and an fp32 MFMA instruction execute together,
// so every vector instruction there takes MFMA time).
#ifndef LCMA_LITERAL_STAGE
#define LCMA_LITERAL_STAGE 1
#endif
template <class T> constexpr bool LITERAL_STAGE = LCMA_LITERAL_STAGE != 0;
template <bool LIT, class F> LCMA_DEV void stage_loop(int y0, int y1, F step) { // y0 even
    if constexpr (LIT) {
        int y = y0;
        for (; y + 1 < y1; y += 2) {
            step(y, 0);
            step(y + 1, 1);
        }
        if (y < y1) step(y, 0);
    } else {
        for (int y = y0; y < y1; ++y) step(y, y & 1);
    }
}

// The y loop of Algorithm 2 for one chunk over two LDS stages.
//
// Ragged K: only the loads of the last y steps can reach past K.  The loop is therefore run in two
// parts, the steps whose loads stay inside K without any guard code and the few tail steps with the
// guard on the A loads (the guard cost 4 % when it sat in every step).  main_steps(D, G) is where the
// tail begins for a loop that loads tile y + D in step y, rounded down to a multiple of G stages.
template <class T> LCMA_DEV int main_steps(const Ctx<T> &cx, int D, int G) {
    const int yt = (int)(cx.p.k_tail_b / (T::TK * T::ES)); // first tile that reaches past K (ny if none)
    const int m = yt - D > 0 ? yt - D : 0;
    return m / G * G;
}

template <class T, class CH> LCMA_DEV void run_chunk(const Ctx<T> &cx, typename T::Acc (&acc)[CH::NP]) {
    const int ny = cx.p.ny, last = ny - 1;
    if constexpr (T::FC) {
        static_assert(CH::NA <= T::NSA && (T::PB ? CH::NP : CH::NB) <= T::NSB, "blocks exceed the LDS slots");
        const FlatStage<T, CH> fs(cx);
        if constexpr (T::PIPE == 0) {
            typename FlatStage<T, CH>::Raw r;
            fs.issue(cx, r, 0, true);
            auto make_step = [&](auto guard) {
                return [&](int y, int st) {
                    fs.store(cx, r, st);
                    fs.issue(cx, r, y + 1 < ny ? y + 1 : last, decltype(guard)::value);
                    __syncthreads();
                    cx.template mma_stage_fc<CH>(st, acc);
                };
            };
            const int ym = main_steps(cx, 1, 2);
            stage_loop<LITERAL_STAGE<T>>(0, ym, make_step(std::false_type{}));
            stage_loop<LITERAL_STAGE<T>>(ym, ny, make_step(std::true_type{}));
            __syncthreads();
        } else if constexpr (T::DL && T::TB) {
            // Direct loads of both raw operands, three LDS stages: the tiles of step y+2 travel into stage
            // (y+2)%3 while step y is multiplied out of stage y%3, a piece (one work-group load instruction)
            // after each product group.  At the end of a step a wave waits only for its loads of step y+1:
            // the newest batch stays in flight across the barrier, so a load has two steps to arrive.
            using DS = DirectStage<T, CH>;
            static_assert(DS::NCA % T::NT == 0 && DS::NCB % T::NT == 0, "every wave issues every piece, so that the count of loads in flight is known");
            static_assert(T::NKK % 2 == 0, "fragment buffers must return to buffer 0 at the end of a step");
            const DS dl(cx);
            dl.issue(cx, 0, 0);
            dl.issue(cx, 1, ny > 1 ? 1 : last);
            DS::template barrier_keeping<DS::NPIECE>();
            auto make_step = [&](auto guard) {
                return [&](int y, int st) { // st = y % 3, a literal at every call site
                    const int nxt = y + 2 < ny ? y + 2 : last; // past the end: the last tile again, unused
                    direct_load_step<T, CH, decltype(guard)::value>(cx, dl, cx.lds + st * T::STAGE,
                                                                    cx.lds + ((st + 2) % 3) * T::STAGE, nxt, acc);
                    DS::template barrier_keeping<DS::NPIECE>();
                };
            };
            auto loop3 = [&](int y0, int y1, auto step) { // y0 a multiple of 3
                int y = y0;
                for (; y + 2 < y1; y += 3) {
                    step(y, 0);
                    step(y + 1, 1);
                    step(y + 2, 2);
                }
                if (y < y1) step(y, 0);
                if (y + 1 < y1) step(y + 1, 1);
            };
            const int ym = main_steps(cx, 2, 3);
            loop3(0, ym, make_step(std::false_type{}));
            loop3(ym, ny, make_step(std::true_type{}));
            DS::landed(); // the loads issued by the last steps must not land on the epilogue's use of LDS
            __syncthreads();
        } else if constexpr (T::DL) {
            // Direct loads: the tiles of step y+1 travel into the other stage while step y is multiplied;
            // a piece (one work-group load instruction) is issued after each product group.
            const DirectStage<T, CH> dl(cx);
            dl.issue(cx, 0, 0);
            dl.landed();
            __syncthreads();
            auto make_step = [&](auto guard) {
                return [&](int y, int st) {
                    const int nxt = y + 1 < ny ? y + 1 : last; // past the end: the last tile again, unused
                    using DS = DirectStage<T, CH>;
                    cx.template mma_stage_pb<CH>(st, acc, [&](int slot, int slots) {
#pragma unroll
                        for (int pc = 0; pc < DS::NPIECE; ++pc)
                            if (pc * slots / DS::NPIECE == slot) {
                                __builtin_amdgcn_sched_barrier(0);
                                dl.issue_piece(cx, pc, st ^ 1, nxt, decltype(guard)::value);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                    });
                    dl.landed();
                    __syncthreads();
                };
            };
            const int ym = main_steps(cx, 1, 2);
            stage_loop<LITERAL_STAGE<T>>(0, ym, make_step(std::false_type{}));
            stage_loop<LITERAL_STAGE<T>>(ym, ny, make_step(std::true_type{}));
        } else if constexpr (T::PIPE == 2 && T::STAGES == 3) {
            // As below, with a third LDS stage: step y multiplies stage y%3, writes tile y+2 into stage
            // (y+2)%3 and reloads the registers with tile y+3.  The stage of step y+1 is complete one
            // barrier earlier than it is needed, so its first fragments are read under the last MFMAs
            // of step y and no wave starts a step by waiting for LDS.
            static_assert(T::NKK % 2 == 0, "fragment buffers must return to buffer 0 at the end of a step");
            using FS = FlatStage<T, CH>;
            typename FS::Raw r;
            fs.issue(cx, r, 0, true);
            fs.store(cx, r, 0);
            fs.issue(cx, r, ny > 1 ? 1 : last, true);
            fs.store(cx, r, 1);
            fs.issue(cx, r, ny > 2 ? 2 : last, true);
            __syncthreads();
            typename Ctx<T>::template Frags<CH> f;
            cx.template fetch_frags<CH>(f, 0, 0, 0);
            auto make_step = [&](auto guard) {
                return [&](int y, int st) { // st = y % 3, a literal at every call site
                    const int nxt = y + 3 < ny ? y + 3 : last; // past the end: reload the last tile, unused
                    cx.template mma_stage_fc<CH>(st, (st + 1) % 3, f, acc, [&](int slot, int slots) {
#pragma unroll
                        for (int pc = 0; pc < FS::NPIECE; ++pc)
                            if (pc * slots / FS::NPIECE == slot) {
                                __builtin_amdgcn_sched_barrier(0);
                                fs.store_piece(cx, r, pc, (st + 2) % 3);
                                fs.issue_piece(cx, r, pc, nxt, decltype(guard)::value);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                    });
                    __syncthreads();
                };
            };
            auto loop3 = [&](int y0, int y1, auto step) { // y0 a multiple of 3
                int y = y0;
                for (; y + 2 < y1; y += 3) {
                    step(y, 0);
                    step(y + 1, 1);
                    step(y + 2, 2);
                }
                if (y < y1) step(y, 0);
                if (y + 1 < y1) step(y + 1, 1);
            };
            const int ym = main_steps(cx, 3, 3);
            loop3(0, ym, make_step(std::false_type{}));
            loop3(ym, ny, make_step(std::true_type{}));
        } else if constexpr (T::PIPE == 2) {
            // Staging spread over the MFMA phase: while step y is multiplied out of one LDS stage, each
            // thread writes its pieces of step y+1 to the other stage and reloads the piece's registers
            // with step y+2, a piece at a time between product groups, so that the LDS writes and the
            // buffer loads issue under executing MFMAs.  One barrier per step: the stage written during
            // step y was last read in step y-1, before the previous barrier.
            using FS = FlatStage<T, CH>;
            typename FS::Raw r;
            fs.issue(cx, r, 0, true);
            fs.store(cx, r, 0);
            fs.issue(cx, r, ny > 1 ? 1 : 0, true);
            __syncthreads();
            auto make_step = [&](auto guard) {
                return [&](int y, int st) {
                    const int nxt = y + 2 < ny ? y + 2 : last; // past the end: reload the last tile, unused
                    auto hook = [&](int slot, int slots) {
#pragma unroll
                        for (int pc = 0; pc < FS::NPIECE; ++pc)
                            if (pc * slots / FS::NPIECE == slot) {
                                __builtin_amdgcn_sched_barrier(0);
                                fs.store_piece(cx, r, pc, st ^ 1);
                                fs.issue_piece(cx, r, pc, nxt, decltype(guard)::value);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                    };
                    if constexpr (T::PB) cx.template mma_stage_pb<CH>(st, acc, hook);
                    else cx.template mma_stage_fc<CH>(st, acc, hook);
                    __syncthreads();
                };
            };
            const int ym = main_steps(cx, 2, 2);
            stage_loop<LITERAL_STAGE<T>>(0, ym, make_step(std::false_type{}));
            stage_loop<LITERAL_STAGE<T>>(ym, ny, make_step(std::true_type{}));
        }
    } else {
        static_assert(T::PIPE == 0, "staged-combine kernels stage in one phase");
        // Plain double buffering: one register set, loads of step y+1 in flight during the MFMAs
        // of step y.  Meant for two work-groups per CU, which overlap each other's phases.
        RawSet<T, CH> r;
        issue_loads<T, CH>(cx, r, 0, true);
        auto make_step = [&](auto guard) {
            return [&](int y, int st) {
                combine_store<T, CH>(cx, r, st);
                issue_loads<T, CH>(cx, r, y + 1 < ny ? y + 1 : last, decltype(guard)::value);
                __syncthreads();
                mma_step<T, CH>(cx, st, acc);
            };
        };
        const int ym = main_steps(cx, 1, 2);
        stage_loop<LITERAL_STAGE<T>>(0, ym, make_step(std::false_type{}));
        stage_loop<LITERAL_STAGE<T>>(ym, ny, make_step(std::true_type{}));
        __syncthreads();
    }
}

} // namespace lcma
