// Device-side building blocks of the fused LCMA kernel for gfx950 (CDNA4, 64-wide waves).
//
// One work-group (4 waves) owns one GROUP in the sense of the paper's Group-Parallel
// Optimization (Sec. 3.2, Algorithm 2): the tile at coordinate (x, z) of every block of C.
// The R products of the scheme are cut into CHUNKS.  For a chunk the work-group walks y
// (the K/k direction): it loads the tiles A_{i,l}[x,y], B_{l,j}[y,z] that the chunk needs
// (coalesced 16-byte buffer loads), forms the chunk's operand combinations of Eq. 3 / Eq. 4
// in registers, writes them to LDS (never to HBM) and multiplies them with MFMA into one fp32
// accumulator tile per product (Eq. 5).  After the chunk, the generated code applies W
// (Eq. 6) in fp32 registers.  Everything that depends on U, V, W is straight-line generated
// code (Sec. 3.1, coefficients as compile-time constants); this header is scheme-agnostic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_params.h"

namespace lcma {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define LCMA_LDS __attribute__((address_space(3)))
#define LCMA_DEV __device__ __forceinline__

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
};

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
// WGM x WGN: wave grid (4 waves); NSLOT: products whose combinations are resident per stage;
// STAGES: LDS stages.
template <class IN_, class CT_, int TM_, int TN_, int TK_, int WGM_, int WGN_, int NSLOT_, int STAGES_, int PIPE_ = 0>
struct Tile {
    static constexpr int PIPE = PIPE_; // 0: double-buffered phases, 1: software-pipelined step
    using IN = IN_;
    using CT = CT_;
    static_assert(IN::ES == CT::ES, "conversion must keep the element size");
    static constexpr int TM = TM_, TN = TN_, TK = TK_, WGM = WGM_, WGN = WGN_;
    static constexpr int NSLOT = NSLOT_, STAGES = STAGES_;
    static constexpr int ES = CT::ES, CH = CT::CH;
    static constexpr int NT = 64 * WGM * WGN;
    static constexpr int WM = TM / WGM, WN = TN / WGN;
    static constexpr int NMI = WM / 32, NNI = WN / 32;
    static constexpr int KSTEP = (ES == 2) ? 16 : 8; // k covered by one fragment read
    static constexpr int NKK = TK / KSTEP;
    static constexpr int CPR_A = TK / CH, CPR_B = TN / CH; // 16-byte chunks per LDS row
    static constexpr int NCHK_A = TM * CPR_A, NCHK_B = TK * CPR_B;
    static constexpr int QA = (NCHK_A + NT - 1) / NT, QB = (NCHK_B + NT - 1) / NT;
    static constexpr int A_ROW = TK * ES, B_ROW = TN * ES; // LDS row pitch in bytes
    static constexpr int A_SLOT = TM * A_ROW, B_SLOT = TK * B_ROW;
    static constexpr int A_STAGE = NSLOT * A_SLOT, B_STAGE = NSLOT * B_SLOT;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int LDS_BYTES = STAGES * STAGE;
    static_assert(NT == 256, "four waves per work-group");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && TK % KSTEP == 0, "MFMA 32x32 tiling");
    static_assert(TK % CH == 0 && TN % CH == 0, "16-byte chunks");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");

    struct Acc {
        f32x16 v[NMI][NNI];
    };

    // LDS swizzles: XOR on the 16-byte chunk index of a row.
    // A rows are read 16 rows at a time (one chunk column): spread them over the 16 chunk
    // positions of a 256-byte bank window.
    static LCMA_DEV constexpr int swz_a(int row, int c) {
        constexpr int rpw = (CPR_A >= 16) ? 1 : 16 / CPR_A; // rows per 256-byte window
        constexpr int mask = (CPR_A >= 16) ? 15 : CPR_A - 1;
        return c ^ ((row / rpw) & mask);
    }
    // B rows are read four k-rows at a time, 64 bytes from each (16-bit types): move the four
    // rows to four different 64-byte segments of the bank window.
    static LCMA_DEV constexpr int swz_b(int row, int c) {
        if constexpr (ES == 2) {
            if constexpr (CPR_B >= 16) return c ^ ((row & 3) << 2);
            else if constexpr (CPR_B == 8) return c ^ (((row >> 1) & 1) << 2);
            else return c;
        } else {
            if constexpr (CPR_B >= 16) return c ^ (((row >> 2) & 1) << 3);
            else return c;
        }
    }
};

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
    static LCMA_DEV void run(const frag &a, const frag &b, f32x16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<BF16> {
    using frag = bf16x8;
    static LCMA_DEV void run(const frag &a, const frag &b, f32x16 &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<F32> {
    using frag = f32x4;
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
    uint32_t a_voff[T::QA], b_voff[T::QB];
    uint32_t a_lds[T::QA], b_lds[T::QB];
    uint32_t a_frag[T::NKK], b_frag[T::NNI];
    uint32_t c_voff; // byte offset of this lane's first output element inside the tile

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
        const int total = p.nx * p.nz;
        int id = blockIdx.x;
        const int per = total >> 3;
        if (id < (per << 3)) id = (id & 7) * per + (id >> 3);
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
        b_group = (uint32_t)z * T::TN * T::ES;
        c_group = (uint32_t)x * T::TM * p.ldc_b + (uint32_t)z * T::TN * T::ES;

#pragma unroll
        for (int q = 0; q < T::QA; ++q) {
            // a tile smaller than the work-group is staged twice by threads that wrap around
            // (same data to the same address), which keeps the pipeline free of branches
            const int id2 = (q * T::NT + tid) % T::NCHK_A;
            const int row = id2 / T::CPR_A, c = id2 % T::CPR_A;
            a_voff[q] = (uint32_t)row * p.lda_b + c * 16;
            a_lds[q] = row * T::A_ROW + T::swz_a(row, c) * 16;
        }
#pragma unroll
        for (int q = 0; q < T::QB; ++q) {
            const int id2 = (q * T::NT + tid) % T::NCHK_B;
            const int row = id2 / T::CPR_B, c = id2 % T::CPR_B;
            b_voff[q] = (uint32_t)row * p.ldb_b + c * 16;
            b_lds[q] = T::A_STAGE + row * T::B_ROW + T::swz_b(row, c) * 16;
        }
        // Fragment addresses.  A operand of the 32x32 MFMA: lane holds row lane%32 and the
        // (lane/32)-th group of consecutive k -> one 16-byte read.
        const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < T::NKK; ++kk) {
            const int row = wm * T::WM + l32;
            a_frag[kk] = row * T::A_ROW + T::swz_a(row, kk * 2 + lh) * 16;
        }
        if constexpr (T::ES == 2) {
            // B operand, 16-bit: column lane%32, 8 consecutive k.  The tile is stored
            // n-contiguous, so it is read with the transposing 64-bit LDS load: 16 lanes
            // fetch a 4(k) x 16(n) patch (lane i supplies row i/4, columns 4*(i%4)..+3) and
            // lane j receives column j.
            const int i16 = lane & 15, g = (lane >> 4) & 1;
#pragma unroll
            for (int ni = 0; ni < T::NNI; ++ni) {
                const int row = 8 * lh + (i16 >> 2);
                const int col = wn * T::WN + ni * 32 + 16 * g + 4 * (i16 & 3);
                b_frag[ni] = T::A_STAGE + row * T::B_ROW + T::swz_b(row, col >> 3) * 16 + ((col >> 2) & 1) * 8;
            }
        } else {
            // fp32: lane reads B[k][n = lane%32] for k = 4*(lane/32) + t, one dword each.
#pragma unroll
            for (int ni = 0; ni < T::NNI; ++ni) {
                const int row = 4 * lh;
                const int col = wn * T::WN + ni * 32 + l32;
                b_frag[ni] = T::A_STAGE + row * T::B_ROW + T::swz_b(row, col >> 2) * 16 + (col & 3) * 4;
            }
        }
        // Output: accumulator register v of MFMA tile (mi, ni) is row 8*(v/4) + 4*(lane/32) + v%4,
        // column lane%32 of that 32x32 tile.
        c_voff = (uint32_t)(wm * T::WM + 4 * lh) * p.ldc_b + (uint32_t)(wn * T::WN + l32) * T::ES;
    }

    LCMA_DEV u32x4 load_a(int q, uint32_t soff) const {
        return __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_voff[q], (int)soff, 0);
    }
    LCMA_DEV u32x4 load_b(int q, uint32_t soff) const {
        return __builtin_amdgcn_raw_buffer_load_b128(rb, (int)b_voff[q], (int)soff, 0);
    }
    // Scalar byte offset of tile y of block A_{i,l} / B_{l,j} for this group.
    LCMA_DEV uint32_t soff_a(int i, int l, int y) const {
        return (uint32_t)i * p.a_brow + (uint32_t)l * p.a_bcol + a_group + (uint32_t)y * (T::TK * T::ES);
    }
    LCMA_DEV uint32_t soff_b(int l, int j, int y) const {
        return (uint32_t)l * p.b_brow + (uint32_t)j * p.b_bcol + b_group + (uint32_t)y * T::TK * p.ldb_b;
    }

    LCMA_DEV void lds_store(uint32_t off, const V &v) const {
        *(LCMA_LDS u32x4 *)(lds + off) = __builtin_bit_cast(u32x4, v);
    }

    // acc[s] += At_s x Bt_s for the NP products resident in LDS stage `st`.
    template <int NP> LCMA_DEV void mma_stage(int st, typename T::Acc (&acc)[NP]) const {
        const uint32_t sb = st * T::STAGE;
#pragma unroll
        for (int s = 0; s < NP; ++s) {
#pragma unroll
            for (int kk = 0; kk < T::NKK; ++kk) {
                Frag a[T::NMI], b[T::NNI];
#pragma unroll
                for (int mi = 0; mi < T::NMI; ++mi)
                    a[mi] = __builtin_bit_cast(
                        Frag, *(LCMA_LDS u32x4 *)(lds + sb + s * T::A_SLOT + a_frag[kk] + mi * 32 * T::A_ROW));
#pragma unroll
                for (int ni = 0; ni < T::NNI; ++ni) {
                    const uint32_t base = sb + s * T::B_SLOT + b_frag[ni] + kk * T::KSTEP * T::B_ROW;
                    if constexpr (T::ES == 2) {
                        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LCMA_LDS i16x4 *)(lds + base));
                        const i16x4 hi =
                            __builtin_amdgcn_ds_read_tr16_b64_v4i16((LCMA_LDS i16x4 *)(lds + base + 4 * T::B_ROW));
                        i16x8 both;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            both[e] = lo[e];
                            both[e + 4] = hi[e];
                        }
                        b[ni] = __builtin_bit_cast(Frag, both);
                    } else {
                        f32x4 t;
#pragma unroll
                        for (int e = 0; e < 4; ++e) t[e] = *(LCMA_LDS float *)(lds + base + e * T::B_ROW);
                        b[ni] = t;
                    }
                }
#pragma unroll
                for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < T::NNI; ++ni) Mma<CT>::run(a[mi], b[ni], acc[s].v[mi][ni]);
            }
        }
    }

    // Round and store one fp32 tile into block C_{i,j}.  f(mi, ni) returns the f32x16 of MFMA
    // tile (mi, ni).
    template <class F> LCMA_DEV void store_c(int i, int j, F f) const {
        const uint32_t soff = (uint32_t)i * p.c_brow + (uint32_t)j * p.c_bcol + c_group;
#pragma unroll
        for (int mi = 0; mi < T::NMI; ++mi)
#pragma unroll
            for (int ni = 0; ni < T::NNI; ++ni) {
                const f32x16 t = f(mi, ni);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t off =
                        c_voff + (uint32_t)(mi * 32 + (v >> 2) * 8 + (v & 3)) * p.ldc_b + ni * 32 * T::ES;
                    const uint32_t bits = Round<IN>::run(t[v]);
                    if constexpr (T::ES == 2)
                        __builtin_amdgcn_raw_buffer_store_b16((short)bits, rc, (int)off, (int)soff, 0);
                    else
                        __builtin_amdgcn_raw_buffer_store_b32(bits, rc, (int)off, (int)soff, 0);
                }
            }
    }
};

// ---------------------------------------------------------------- one chunk of products over all y
// CH (generated) describes the chunk:
//   NA, NB, NP        raw A tiles, raw B tiles, products
//   a_i(t), a_l(t)    block indices of raw A tile t; b_l(t), b_j(t) likewise for B
//   comb_a(in, out)   out[s] = sum_t U * in[t]  (Eq. 3) on 16-byte vectors; comb_b likewise (Eq. 4)
template <class T, class CH> struct RawSet {
    u32x4 a[CH::NA][T::QA], b[CH::NB][T::QB];
};

// Issue the buffer loads of step y into `r`.
template <class T, class CH> LCMA_DEV void issue_loads(const Ctx<T> &cx, RawSet<T, CH> &r, int y) {
#pragma unroll
    for (int t = 0; t < CH::NA; ++t) {
        const uint32_t so = cx.soff_a(CH::a_i(t), CH::a_l(t), y);
#pragma unroll
        for (int q = 0; q < T::QA; ++q)
            r.a[t][q] = cx.load_a(q, so);
    }
#pragma unroll
    for (int t = 0; t < CH::NB; ++t) {
        const uint32_t so = cx.soff_b(CH::b_l(t), CH::b_j(t), y);
#pragma unroll
        for (int q = 0; q < T::QB; ++q)
            r.b[t][q] = cx.load_b(q, so);
    }
}

// Convert the raw tiles in `r`, form the chunk's combinations (Eq. 3 / Eq. 4) and write them to LDS
// stage `st`.
template <class T, class CH> LCMA_DEV void combine_store(const Ctx<T> &cx, const RawSet<T, CH> &r, int st) {
    using V = typename T::CT::vec;
    using Cv = Convert<typename T::IN, typename T::CT>;
    const uint32_t sb = st * T::STAGE;
#pragma unroll
    for (int q = 0; q < T::QA; ++q) {
        V in[CH::NA], out[CH::NP];
#pragma unroll
        for (int t = 0; t < CH::NA; ++t) in[t] = Cv::run(r.a[t][q]);
        CH::comb_a(in, out);
#pragma unroll
        for (int s = 0; s < CH::NP; ++s) cx.lds_store(sb + s * T::A_SLOT + cx.a_lds[q], out[s]);
    }
#pragma unroll
    for (int q = 0; q < T::QB; ++q) {
        V in[CH::NB], out[CH::NP];
#pragma unroll
        for (int t = 0; t < CH::NB; ++t) in[t] = Cv::run(r.b[t][q]);
        CH::comb_b(in, out);
#pragma unroll
        for (int s = 0; s < CH::NP; ++s) cx.lds_store(sb + s * T::B_SLOT + cx.b_lds[q], out[s]);
    }
}

// The y loop of Algorithm 2 for one chunk, software-pipelined over two LDS stages and two register
// sets.  In the steady state one step (a single basic block, so that the scheduler may interleave
// its parts) does: issue the loads of step y+2; multiply step y from LDS stage y%2; combine step
// y+1 from registers into the other stage; barrier.  Loads therefore have a whole step of MFMA work
// to arrive, and the additions, conversions and LDS writes share the step with the MFMAs.  Past the
// end the last tile is loaded and combined again into the stage nobody reads, which keeps the
// step branch-free.
template <class T, class CH> LCMA_DEV void run_chunk(const Ctx<T> &cx, typename T::Acc (&acc)[CH::NP]) {
    static_assert(CH::NP <= T::NSLOT, "chunk larger than the LDS slots");
    static_assert(T::STAGES == 2, "two LDS stages");
    const int ny = cx.p.ny, last = ny - 1;
    if constexpr (T::PIPE == 0) {
        // Plain double buffering: one register set, loads of step y+1 in flight during the MFMAs
        // of step y.  Meant for two work-groups per CU, which overlap each other's phases.
        RawSet<T, CH> r;
        issue_loads<T, CH>(cx, r, 0);
        for (int y = 0; y < ny; ++y) {
            combine_store<T, CH>(cx, r, y & 1);
            issue_loads<T, CH>(cx, r, y + 1 < ny ? y + 1 : last);
            __syncthreads();
            cx.template mma_stage<CH::NP>(y & 1, acc);
        }
        __syncthreads();
    } else {
        RawSet<T, CH> r0, r1;
        issue_loads<T, CH>(cx, r0, 0);
        issue_loads<T, CH>(cx, r1, ny > 1 ? 1 : 0);
        combine_store<T, CH>(cx, r0, 0);
        __syncthreads();
        for (int y = 0; y < ny; y += 2) {
            {   // even step: stage 0 holds y, r1 holds y+1, r0 is free
                const int yn = y + 2 < ny ? y + 2 : last;
                issue_loads<T, CH>(cx, r0, yn);
                cx.template mma_stage<CH::NP>(0, acc);
                combine_store<T, CH>(cx, r1, 1);
                __syncthreads();
            }
            if (y + 1 >= ny) break;
            {   // odd step: stage 1 holds y+1, r0 holds y+2, r1 is free
                const int yn = y + 3 < ny ? y + 3 : last;
                issue_loads<T, CH>(cx, r1, yn);
                cx.template mma_stage<CH::NP>(1, acc);
                combine_store<T, CH>(cx, r0, 0);
                __syncthreads();
            }
        }
    }
}

} // namespace lcma
