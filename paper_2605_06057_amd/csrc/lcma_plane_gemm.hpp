// Plane GEMM for gfx950: C = A x W^T on k-contiguous operands (A: M x K rows, W: N x K rows), for FP8 codes with
// E8M0 block scales, fp16 and bf16, plain or batched over the R planes of a scheme (the products H_r = At_r Bt_r of
// Eq. 5 in Algorithm 1), with the work handed out the way the paper's Split-Group Parallelism does (Sec. 3.2).
//
// Data path.  A step is 128 bytes of every row of the tile (128 FP8 or 64 16-bit elements of K), two LDS stages, one
// barrier per step.  Both operands travel from memory straight into LDS (buffer loads with the LDS bit: no staging
// registers, no LDS write instructions; the swizzle is applied by choosing which 16-byte chunk of memory each lane
// fetches): the loads of step y + 1 are issued at the start of step y into the stage that step y - 1 read, and must
// have landed at the barrier that ends step y.  Four things decide the speed of this loop on MI355X (each measured
// in one run against the alternative): the matrix instructions must be pinned above the wait for the loads (they touch
// no memory, so the compiler otherwise sinks them below it and the wait follows the issue of the loads directly:
// -20 %); the scale bytes must come as one dword per four steps, not as a byte load per step (six more vector memory
// instructions per wave and step: -20 %; the vector memory path is the busy one); direct loads beat staging through
// registers (DIRECT = false, kept for comparison) by 6 % for 16-bit operands and 1 % for FP8; and the barrier sits in
// front of the LAST fragment set's matrix instructions, with the first fragment reads of the next step behind it
// (step_across: +4 % on random operands, +6 % on all-zero operands, where the chip's power limit does not hide it).
// Measured and not adopted: a ring of three to five half-step stages (64 bytes of a row each, loads two to four
// half-steps ahead): 5 % slower at every depth, so the distance of the loads is not what bounds the loop; spreading
// the loads between the matrix instructions: no gain; four waves with 128 x 128 wave tiles: 6 % slower.
//
// Scheduling (Sec. 3.2).  The unit of work is one step of one tile-product; all steps of all tile-products are
// numbered tile-product-major (tile-products in product-major order, the paper's Cache-Aware order: work-groups that
// run together share r) and the launch consists of `units` persistent work-groups; work-group u owns the contiguous
// range [u * cap, (u + 1) * cap) with cap = ceil(total / units).  A tile-product may therefore straddle two (or, when
// there are fewer tile-products than work-groups, more) work-groups, exactly like a group straddles two SMs in the
// paper; no atomics are needed because every piece has one owner: a work-group that holds a whole tile-product rounds
// and stores it, a work-group that holds a piece writes its fp32 partial sums to its own slot of a scratch buffer, and
// a second, small kernel adds the pieces of each split tile-product in ascending work-group order and rounds once.
// With units = number of tile-products and cap = steps per tile-product this is the ordinary one-tile-per-work-group
// launch (no piece is ever written).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_device.hpp"

namespace lcma {

typedef int i32x8 __attribute__((ext_vector_type(8)));

struct FP8 { // E4M3 codes; one E8M0 scale byte per row and step
    static constexpr int ES = 1;
};

template <class K> struct PlaneFrag {
    using type = typename Mma<K>::frag;
};
template <> struct PlaneFrag<FP8> {
    using type = i32x8;
};

template <class KIND, int TM, int TN, int WGM, int WGN, class OUT, bool SPLIT = true, bool DIRECT = true> struct PlaneGemm {
    static constexpr int NT = 64 * WGM * WGN, WM = TM / WGM, WN = TN / WGN, NMI = WM / 32, NNI = WN / 32;
    static constexpr int ROW = 128, A_STAGE = TM * ROW, B_STAGE = TN * ROW, STAGE = A_STAGE + B_STAGE;
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int QA = TM * 8 / NT, QB = TN * 8 / NT; // direct-load instructions per thread and step
    static constexpr bool SCALED = std::is_same_v<KIND, FP8>;
    // fragment sets of a step (see read_set)
    static constexpr int SUBS = 4, NA = SCALED ? NMI / 2 : NMI;
    static_assert(!SCALED || NMI % 2 == 0, "FP8: fragment sets of half the tile rows");
    using FragT = typename PlaneFrag<KIND>::type;
    static_assert(TM * 8 % NT == 0 && TN * 8 % NT == 0 && WM % 32 == 0 && WN % 32 == 0, "tile and wave grid");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
    static constexpr int TILE_FLOATS = TM * TN;
    // the persistent kernel sends the first loads of its next tile-product during the last step of the current one when
    // the epilogue's strips fit the one stage that is free by then
    // rows of the strip a wave passes through LDS at a time in the epilogue: 32, or 16 for fp32 output, so that the strips
    // of all waves fit one stage
    static constexpr int STRIP_ROWS = OUT::ES == 4 ? 16 : 32;
    static constexpr bool XTILE = SPLIT && DIRECT && NT / 64 * STRIP_ROWS * (WN * OUT::ES + 16) <= STAGE;

    // 128-byte rows: two rows per 256-byte bank window; 16 consecutive rows at one chunk column spread over the 16
    // chunk positions of a window
    static LCMA_DEV constexpr int swz(int row, int c) { return c ^ ((row >> 1) & 7); }

    // every direct load of this wave has landed, then the waves meet.  __syncthreads() is not used: its fences order
    // the LDS writes of loads in flight as well and would be placed by the compiler where it sees fit.
    // The scheduling barriers keep the matrix instructions of the step above the wait: they touch no memory, so
    // nothing else stops the compiler from sinking them below it, which would put the wait for the loads right
    // behind their issue.
    static LCMA_DEV void landed_barrier() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0070); // vmcnt(0) lgkmcnt(0)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    }

    struct State {
        __amdgpu_buffer_rsrc_t ra, rb, rsa, rsb, rc;
        uint32_t a_voff, b_voff; // of the first direct load of a step; load q is NT / 8 rows further down
        uint32_t a_step, b_step; // byte step between the rows of consecutive loads
        uint32_t a_lds, b_lds;   // register staging: LDS position of this thread's chunk (load q: q * NT / 8 rows further down)
        uint32_t a_frag[2][2], b_frag[2][2];
        int wave_chunk, lane, w, wm, wn, l32, lh;
    };

    // loads of step y of the tile at (a_base, b_base) into the stage at `stage`
    static LCMA_DEV void issue(const State &s, LCMA_LDS char *stage, uint32_t a_base, uint32_t b_base, int y) {
#pragma unroll
        for (int q = 0; q < QA; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(s.ra, (LCMA_LDS void *)(stage + (q * NT + s.wave_chunk) * 16), 16,
                                                     (int)s.a_voff, (int)(a_base + (uint32_t)y * ROW + q * s.a_step), 0, 0);
#pragma unroll
        for (int q = 0; q < QB; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(s.rb, (LCMA_LDS void *)(stage + A_STAGE + (q * NT + s.wave_chunk) * 16), 16,
                                                     (int)s.b_voff, (int)(b_base + (uint32_t)y * ROW + q * s.b_step), 0, 0);
    }

    static LCMA_DEV i32x8 frag8(const LCMA_LDS char *base, uint32_t off0, uint32_t off1) {
        const u32x4 lo = *(const LCMA_LDS u32x4 *)(base + off0), hi = *(const LCMA_LDS u32x4 *)(base + off1);
        return i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }

    // Multiply out of the stage at `rd` while the loads of the next step travel into the stage at `wr` (restrict:
    // the loads in flight do not touch what the fragment reads read, so the compiler need not wait for them).
    static LCMA_DEV void step(const State &s, const LCMA_LDS char *__restrict__ rd, LCMA_LDS char *__restrict__ wr,
                              uint32_t a_base, uint32_t b_base, int y_next, bool more, const int (&sa)[NMI], const int (&sb)[NNI],
                              f32x16 (&acc)[NMI][NNI]) {
        if constexpr (DIRECT) {
            if (more) issue(s, wr, a_base, b_base, y_next);
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            if (SCALED && kk) { // 32-byte fragments: keep those of one half live at a time (register budget)
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (SCALED) {
                i32x8 a[NMI], b[NNI];
#pragma unroll
                for (int mi = 0; mi < NMI; ++mi)
                    a[mi] = frag8(rd, s.a_frag[kk][0] + mi * 32 * ROW, s.a_frag[kk][1] + mi * 32 * ROW);
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni)
                    b[ni] = frag8(rd, s.b_frag[kk][0] + ni * 32 * ROW, s.b_frag[kk][1] + ni * 32 * ROW);
#pragma unroll
                for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NNI; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[mi], b[ni], acc[mi][ni], 0, 0, 0, sa[mi], 0, sb[ni]);
            } else {
                using Frag = typename Mma<KIND>::frag;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    Frag a[NMI], b[NNI];
#pragma unroll
                    for (int mi = 0; mi < NMI; ++mi)
                        a[mi] = __builtin_bit_cast(Frag, *(const LCMA_LDS u32x4 *)(rd + s.a_frag[kk][j] + mi * 32 * ROW));
#pragma unroll
                    for (int ni = 0; ni < NNI; ++ni)
                        b[ni] = __builtin_bit_cast(Frag, *(const LCMA_LDS u32x4 *)(rd + s.b_frag[kk][j] + ni * 32 * ROW));
#pragma unroll
                    for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NNI; ++ni) Mma<KIND>::run(a[mi], b[ni], acc[mi][ni]);
                }
            }
        }
    }

    // Fragment set `sub` of the stage at `st`.  16-bit: the operands of the sub-th 32x32x16 instruction along K for all
    // tiles of the wave (buffers alternate with sub).  FP8: sub = 2 kk + mh, the A fragments of tile rows mh * NA ..
    // of the kk-th 32x32x64 instruction (buffers alternate with sub) and, when mh = 0, the B fragments of kk (buffers
    // alternate with kk): half a set of A at a time keeps two sets in flight inside the register budget.
    static LCMA_DEV void read_set(const State &s, const LCMA_LDS char *st, int sub, FragT (&fa)[2][NA], FragT (&fb)[2][NNI]) {
        if constexpr (SCALED) {
            const int kk = sub >> 1, mh = sub & 1;
#pragma unroll
            for (int i = 0; i < NA; ++i)
                fa[sub & 1][i] = frag8(st, s.a_frag[kk][0] + (mh * NA + i) * 32 * ROW, s.a_frag[kk][1] + (mh * NA + i) * 32 * ROW);
            if (mh == 0) {
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni)
                    fb[kk & 1][ni] = frag8(st, s.b_frag[kk][0] + ni * 32 * ROW, s.b_frag[kk][1] + ni * 32 * ROW);
            }
        } else {
            const int kk = sub >> 1, j = sub & 1;
#pragma unroll
            for (int mi = 0; mi < NMI; ++mi)
                fa[sub & 1][mi] = __builtin_bit_cast(FragT, *(const LCMA_LDS u32x4 *)(st + s.a_frag[kk][j] + mi * 32 * ROW));
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni)
                fb[sub & 1][ni] = __builtin_bit_cast(FragT, *(const LCMA_LDS u32x4 *)(st + s.b_frag[kk][j] + ni * 32 * ROW));
        }
    }

    static LCMA_DEV void mma_set(int sub, const FragT (&fa)[2][NA], const FragT (&fb)[2][NNI], const int (&sa)[NMI],
                                 const int (&sb)[NNI], f32x16 (&acc)[NMI][NNI]) {
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni) {
                if constexpr (SCALED) {
                    const int mi = (sub & 1) * NA + i;
                    acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[sub & 1][i], fb[(sub >> 1) & 1][ni], acc[mi][ni], 0, 0,
                                                                                   0, sa[mi], 0, sb[ni]);
                } else {
                    Mma<KIND>::run(fa[sub & 1][i], fb[sub & 1][ni], acc[i][ni]);
                }
            }
    }

    // One step of the direct-load pipeline.  On entry fa[0], fb[0] hold fragment set 0 of the stage at `rd`; the barrier
    // that ends the step sits in front of the matrix instructions of the LAST fragment set, and the reads of set 0 of
    // the next step (from `wr`, whose loads have landed by then) are issued behind it: the matrix pipe has the last
    // set to work on while those reads travel, where otherwise all waves of a SIMD would stand at the start of a step
    // waiting for their first fragments.  The barrier therefore means "every wave has READ the stage", which is all
    // the next loads into it need.  (restrict: the loads in flight towards `wr` do not touch what is read from `rd`.)
    // a_next / b_next: byte offsets in the operands of the step whose loads leave now (the next step of this
    // tile-product, or the first step of the work-group's next one), if `more`.
    static LCMA_DEV void step_across(const State &s, const LCMA_LDS char *__restrict__ rd, LCMA_LDS char *__restrict__ wr,
                                     uint32_t a_next, uint32_t b_next, bool more, const int (&sa)[NMI],
                                     const int (&sb)[NNI], f32x16 (&acc)[NMI][NNI], FragT (&fa)[2][NA], FragT (&fb)[2][NNI]) {
        if (more) issue(s, wr, a_next, b_next, 0);
        // the loads leave FIRST (the compiler otherwise rotates the loop and sends them half a step later, behind two
        // fragment sets: they then land late and the wait at the barrier grows; measured -14 % on all-zero operands)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int sub = 0; sub + 1 < SUBS; ++sub) {
            read_set(s, rd, sub + 1, fa, fb);
            mma_set(sub, fa, fb, sa, sb, acc);
            // FP8: no reads of later sets above this line (the scheduler would hoist them all and run out of registers)
            if constexpr (SCALED) __builtin_amdgcn_sched_barrier(0);
        }
        landed_barrier();
        // (unconditional on purpose: after the last step this reads a stage nobody uses, and a branch here would let
        // the compiler move the matrix instructions above to this side of the barrier)
        read_set(s, wr, 0, fa, fb);
        // the reads stay here, in front of the last set's matrix instructions (they would otherwise be moved to the
        // top of the next step, behind them)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        mma_set(SUBS - 1, fa, fb, sa, sb, acc);
    }

    static LCMA_DEV void run(const PlaneGemmParams &p, LCMA_LDS char *lds) {
        State s;
        const int tid = threadIdx.x;
        s.lane = tid & 63;
        s.w = tid >> 6;
        s.wm = s.w / WGN;
        s.wn = s.w % WGN;
        s.l32 = s.lane & 31;
        s.lh = s.lane >> 5;
        s.wave_chunk = __builtin_amdgcn_readfirstlane(tid & ~63);
        s.ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.A), 0, (int)p.a_bytes, 0x00020000);
        s.rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.B), 0, (int)p.b_bytes, 0x00020000);
        s.rsa = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.SA), 0, (int)p.sa_bytes, 0x00020000);
        s.rsb = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.SB), 0, (int)p.sb_bytes, 0x00020000);
        s.rc = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)p.c_bytes, 0x00020000);
        // direct loads: LDS position (row, cs) of a stage is filled from memory chunk swz(row, cs) of that row (the XOR
        // is its own inverse); a wave instruction fills 64 consecutive positions
        // (load q of a thread covers row q * NT / 8 + tid / 8 at position tid % 8; NT / 8 is a multiple of 16, so the
        // swizzle is the same for every q and one vector offset serves all loads of an operand)
        {
            const int row = tid >> 3, cs = tid & 7;
            s.a_voff = (uint32_t)row * p.lda_b + swz(row, cs) * 16;
            s.b_voff = (uint32_t)row * p.ldb_b + swz(row, cs) * 16;
            s.a_step = (uint32_t)(NT / 8) * p.lda_b;
            s.b_step = (uint32_t)(NT / 8) * p.ldb_b;
            if constexpr (!DIRECT) { // memory chunk cs of the row goes to LDS position swz(row, cs)
                s.a_voff = (uint32_t)row * p.lda_b + cs * 16;
                s.b_voff = (uint32_t)row * p.ldb_b + cs * 16;
                s.a_lds = row * ROW + swz(row, cs) * 16;
                s.b_lds = A_STAGE + row * ROW + swz(row, cs) * 16;
            }
        }
        // fragments of half kk (64 bytes of a row).  FP8: lane (row, h) takes the 32 bytes at chunks 2h, 2h + 1 for
        // one 32x32x64 instruction; 16-bit: chunk j * 2 + h feeds the j-th 32x32x16 instruction.  Both operands use
        // the same assignment of k to lanes, which is all the product needs.
        const int ar = s.wm * WM + s.l32, br = s.wn * WN + s.l32;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = SCALED ? kk * 4 + s.lh * 2 + j : kk * 4 + j * 2 + s.lh;
                s.a_frag[kk][j] = ar * ROW + swz(ar, c) * 16;
                s.b_frag[kk][j] = A_STAGE + br * ROW + swz(br, c) * 16;
            }

        const int tiles = p.nx * p.nz, ny = p.ny;
        const int total = p.jobs * ny; // the host keeps it below 2^31
        // hardware deals work-groups to the 8 XCDs round-robin: renumber them so that each XCD (with its private L2)
        // holds a contiguous run of ranges, i.e. neighbouring tiles
        int unit = blockIdx.x;
        const int per = p.units >> 3;
        if (unit < (per << 3)) unit = (unit & 7) * per + (unit >> 3);
        const int cap = (int)p.cap, begin = unit * cap, end = begin + cap < total ? begin + cap : total;
        // the pieces of this work-group, in order: steps [y0, y1) of tile-product `job`
        struct Piece {
            int job, y0, y1;
            bool ok;
        };
        auto piece_from = [&](int pos) { // ranges of steps: the piece that starts at step `pos`
            if (pos >= end) return Piece{0, 0, 0, false};
            const int job = pos / ny;
            return Piece{job, pos - job * ny, (job + 1) * ny <= end ? ny : end - job * ny, true};
        };
        // whole tile-products in turn, two ways of dealing them to the XCDs (p.interleave; measured, FFN shapes):
        //  1  rounds: the work-groups running at one time take `units` consecutive tile-products, 32 consecutive ones per
        //     XCD.  All XCDs then work inside the same plane of a batch, whose operands stay in the Infinity Cache for all of
        //     them: the batched stage of Algorithm 1 is 5 % faster this way than with 2;
        //  2  each XCD owns a contiguous eighth of the tile-products (as in the launch with a work-group per tile-product)
        //     and its work-groups take every (units / 8)-th of them.  For a single large product 1 is markedly slower
        //     (all eight XCDs ask the memory side for the same rows at the same time: -17 % on all-zero operands).
        //     The tile-products of the last, partial round are dealt work-group by work-group instead, i.e. evenly over the
        //     XCDs (by 32s they would keep two XCDs busy and leave six idle: 448 tile-products of 4096^3 ran 5 % slower than
        //     with a work-group each).
        const int xcd_jobs = (p.jobs + 7) >> 3, turn = p.interleave == 2 ? p.units >> 3 : p.units;
        const int turn_lo = p.interleave == 2 ? (int)(blockIdx.x & 7) * xcd_jobs : 0;
        const int turn_hi = p.interleave == 2 && turn_lo + xcd_jobs < p.jobs ? turn_lo + xcd_jobs : p.jobs;
        const int whole_rounds = p.jobs / p.units * p.units; // tile-products in whole rounds (1)
        auto in_round = [&](int base) { return base + (p.interleave == 1 && base >= whole_rounds ? (int)blockIdx.x : unit); };
        const int turn_first = p.interleave == 2 ? turn_lo + (int)(blockIdx.x >> 3) : in_round(0);
        auto first_piece = [&]() {
            if constexpr (!SPLIT) return Piece{unit, 0, ny, true}; // one work-group per tile-product
            if (p.interleave) return Piece{turn_first, 0, ny, turn_first < turn_hi};
            return piece_from(begin);
        };
        auto piece_after = [&](const Piece &c) {
            if constexpr (!SPLIT) return Piece{0, 0, 0, false};
            if (p.interleave == 2) return Piece{c.job + turn, 0, ny, c.job + turn < turn_hi};
            if (p.interleave) {
                const int job = in_round((c.job / p.units + 1) * p.units);
                return Piece{job, 0, ny, job < p.jobs};
            }
            return piece_from(c.job * ny + c.y1);
        };
        // tile of a job: product-major; inside a product tiles run down x inside column panels of `panel` z tiles
        auto locate = [&](int job, int &plane, int &x, int &z) {
            plane = job / tiles;
            const int id = job - plane * tiles;
            const int pw = p.panel, full = (p.nz / pw) * pw * p.nx;
            if (id < full) {
                const int pi = id / (pw * p.nx), rem = id - pi * (pw * p.nx);
                x = rem / pw;
                z = pi * pw + rem % pw;
            } else {
                const int w2 = p.nz - (p.nz / pw) * pw, rem = id - full;
                x = rem / w2;
                z = (p.nz / pw) * pw + rem % w2;
            }
        };
        FragT fa[2][NA], fb[2][NNI]; // fragment sets in flight (direct loads); set 0 of a primed piece is read before its loop
        int st = 0;                  // stage that holds the first step of the coming piece
        bool primed = false;         // ... whose loads were sent during the last step of the piece before
        Piece cur = first_piece();
        while (cur.ok) {
            const int y0 = cur.y0, y1 = cur.y1;
            int plane, x, z;
            locate(cur.job, plane, x, z);
            Piece nxt{0, 0, 0, false};
            uint32_t a_first = 0, b_first = 0; // first step of the next piece
            if constexpr (XTILE) {
                nxt = piece_after(cur);
                if (nxt.ok) {
                    int pl, nx_, nz_;
                    locate(nxt.job, pl, nx_, nz_);
                    a_first = (uint32_t)pl * p.a_plane + (uint32_t)nx_ * TM * p.lda_b + (uint32_t)nxt.y0 * ROW;
                    b_first = (uint32_t)pl * p.b_plane + (uint32_t)nz_ * TN * p.ldb_b + (uint32_t)nxt.y0 * ROW;
                }
            }
            const uint32_t a_base = (uint32_t)plane * p.a_plane + (uint32_t)x * TM * p.lda_b;
            const uint32_t b_base = (uint32_t)plane * p.b_plane + (uint32_t)z * TN * p.ldb_b;
            // scale bytes of this lane's rows: one dword holds four consecutive steps and is loaded a group ahead (a byte
            // load per row and step costs a fifth of the kernel's speed: the vector memory path is the busy one)
            const uint32_t sa_base = (uint32_t)plane * p.sa_plane + (uint32_t)(x * TM + ar) * p.lsa_b;
            const uint32_t sb_base = (uint32_t)plane * p.sb_plane + (uint32_t)(z * TN + br) * p.lsb_b;
            uint32_t sa_cur[NMI], sb_cur[NNI], sa_nxt[NMI], sb_nxt[NNI];
            auto load_scales = [&](int g, uint32_t (&da)[NMI], uint32_t (&db)[NNI]) {
                if constexpr (SCALED) {
#pragma unroll
                    for (int mi = 0; mi < NMI; ++mi)
                        da[mi] = __builtin_amdgcn_raw_buffer_load_b32(s.rsa, (int)(sa_base + (uint32_t)mi * 32 * p.lsa_b), g * 4, 0);
#pragma unroll
                    for (int ni = 0; ni < NNI; ++ni)
                        db[ni] = __builtin_amdgcn_raw_buffer_load_b32(s.rsb, (int)(sb_base + (uint32_t)ni * 32 * p.lsb_b), g * 4, 0);
                }
            };
            // before the barrier of step y: new group of four steps?  (uniform branch)
            auto turn_scales = [&](int y) {
                if constexpr (SCALED) {
                    if ((y & 3) == 0 && y > y0) {
#pragma unroll
                        for (int mi = 0; mi < NMI; ++mi) sa_cur[mi] = sa_nxt[mi];
#pragma unroll
                        for (int ni = 0; ni < NNI; ++ni) sb_cur[ni] = sb_nxt[ni];
                        load_scales((y >> 2) + 1, sa_nxt, sb_nxt);
                    }
                }
            };
            auto scales_of = [&](int y, int (&sa)[NMI], int (&sb)[NNI]) {
                if constexpr (SCALED) {
                    const int sh = (y & 3) * 8;
#pragma unroll
                    for (int mi = 0; mi < NMI; ++mi) sa[mi] = (int)((sa_cur[mi] >> sh) & 0xffu);
#pragma unroll
                    for (int ni = 0; ni < NNI; ++ni) sb[ni] = (int)((sb_cur[ni] >> sh) & 0xffu);
                }
            };
            f32x16 acc[NMI][NNI];
#pragma unroll
            for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni) zero(acc[mi][ni]);

            load_scales(y0 >> 2, sa_cur, sb_cur);
            load_scales((y0 >> 2) + 1, sa_nxt, sb_nxt);
            if constexpr (SCALED && XTILE) {
                // the scale dwords are waited for here, once per piece: with these loads still counted as in flight at the
                // top of the step loop the compiler puts a wait for them behind the direct loads of EVERY step, which then
                // waits for two of those as well (the counter runs in order)
                __builtin_amdgcn_s_waitcnt(0x0070);
                asm volatile("" ::: "memory");
            }
            if constexpr (DIRECT) {
                if (!primed) {
                    issue(s, lds + st * STAGE, a_base, b_base, y0);
                    landed_barrier();
                    read_set(s, lds + st * STAGE, 0, fa, fb);
                }
                // the stage alternates and stays a run-time value: two unrolled copies with literal stages gain nothing
                // for 16-bit operands and cost the FP8 kernel 10 % (registers)
                for (int y = y0; y < y1; ++y) {
                    int sa[NMI], sb[NNI];
                    turn_scales(y);
                    scales_of(y, sa, sb);
                    const bool last = y + 1 == y1;
                    step_across(s, lds + st * STAGE, lds + (st ^ 1) * STAGE, last ? a_first : a_base + (uint32_t)(y + 1) * ROW,
                                last ? b_first : b_base + (uint32_t)(y + 1) * ROW, !last || nxt.ok, sa, sb, acc, fa, fb);
                    st ^= 1;
                }
                primed = nxt.ok; // its first step sits in stage st, fragment set 0 of it in fa[0], fb[0]
            } else {
                u32x4 rega[QA], regb[QB];
                auto fetch = [&](int y) {
#pragma unroll
                    for (int q = 0; q < QA; ++q)
                        rega[q] = __builtin_amdgcn_raw_buffer_load_b128(s.ra, (int)s.a_voff, (int)(a_base + (uint32_t)y * ROW + q * s.a_step), 0);
#pragma unroll
                    for (int q = 0; q < QB; ++q)
                        regb[q] = __builtin_amdgcn_raw_buffer_load_b128(s.rb, (int)s.b_voff, (int)(b_base + (uint32_t)y * ROW + q * s.b_step), 0);
                };
                fetch(y0);
                auto one = [&](int y, int st) {
                    LCMA_LDS char *stage = lds + st * STAGE;
#pragma unroll
                    for (int q = 0; q < QA; ++q) *(LCMA_LDS u32x4 *)(stage + s.a_lds + q * (NT / 8) * ROW) = rega[q];
#pragma unroll
                    for (int q = 0; q < QB; ++q) *(LCMA_LDS u32x4 *)(stage + s.b_lds + q * (NT / 8) * ROW) = regb[q];
                    fetch(y + 1 < y1 ? y + 1 : y); // past the end: the last tile again, unused
                    turn_scales(y);
                    // one barrier per step: the stage written now was last read a whole step ago, before the previous barrier
                    __syncthreads();
                    int sa[NMI], sb[NNI];
                    scales_of(y, sa, sb);
                    step(s, stage, stage, a_base, b_base, y + 1, false, sa, sb, acc);
                };
                // the stage alternates from 0 at the first step of the piece
                if constexpr (SPLIT) {
                    // run-time stage: unrolled copies of the step with literal stages cost the persistent kernel more
                    // registers than it has (it spills)
                    for (int y = y0; y < y1; ++y) one(y, (y - y0) & 1);
                } else {
                    // unrolled twice: the stage is a literal at both call sites and every LDS address a register plus an
                    // immediate (worth 5 % here)
                    int y = y0;
                    for (; y + 1 < y1; y += 2) {
                        one(y, 0);
                        one(y + 1, 1);
                    }
                    if (y < y1) one(y, 0);
                }
                __syncthreads(); // the stages are free for the epilogue and for the next tile-product
            }

            // the strips of the epilogue go through the stage the last step read when the other one may already hold the
            // first step of the next piece (they fit one stage then), else through both from the start; every wave has
            // passed the barrier of the last step
            LCMA_LDS char *strips = XTILE ? lds + (st ^ 1) * STAGE : lds;
            if (!SPLIT || (y0 == 0 && y1 == ny)) store_tile(p, s, strips, plane, x, z, acc);
            else store_piece(p, s, unit * 2 + (y0 == 0 ? 1 : 0), acc);
            if constexpr (XTILE) cur = nxt;
            else cur = piece_after(cur);
        }
    }

    // Accumulator value v of tile (mi, ni) is row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32: a lane's values
    // lie in one column.  Each wave passes one strip of STRIP_ROWS rows of its tile at a time through a private piece of
    // LDS (the stages are free: every wave has passed the barrier that ends the last step) and writes it out as 16-byte
    // vectors, whole 128-byte lines.  A strip is private to its wave and a wave's LDS instructions execute in order, so
    // no barrier separates its writes from its reads; one barrier at the end keeps the next loads into these stages
    // behind the last read (eight barriers per tile-product before: the waves no longer wait for each other strip by
    // strip).  The scalar-offset field of these stores stays a literal zero (everything is in the vector offset): the
    // compiler keeps a following vector write at a distance from a store of more than 8 bytes only then.
    static LCMA_DEV void store_tile(const PlaneGemmParams &p, const State &s, LCMA_LDS char *lds, int plane, int x, int z,
                                    const f32x16 (&acc)[NMI][NNI]) {
        constexpr int OES = OUT::ES; // 2: C rounded to fp16 / bf16; 4: the fp32 sums as they are
        constexpr int SR = STRIP_ROWS, PITCH = WN * OES + 16, CPRW = WN * OES / 16, NIT = SR * CPRW / 64;
        static_assert(NT / 64 * SR * PITCH <= (XTILE ? STAGE : LDS_BYTES), "the strips of all waves fit the stage buffers");
        const uint32_t c_base = (uint32_t)plane * p.c_plane + (uint32_t)x * TM * p.ldc_b + (uint32_t)z * TN * OES;
        LCMA_LDS char *strip = lds + s.w * (SR * PITCH);
#pragma unroll
        for (int mi = 0; mi < NMI; ++mi) {
#pragma unroll
            for (int h = 0; h < 32 / SR; ++h) {
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni)
#pragma unroll
                    for (int v = h * (SR / 2); v < (h + 1) * (SR / 2); ++v) {
                        LCMA_LDS char *at = strip + ((v >> 2) * 8 + 4 * s.lh + (v & 3) - h * SR) * PITCH + (ni * 32 + s.l32) * OES;
                        if constexpr (OES == 2) *(LCMA_LDS uint16_t *)at = (uint16_t)Round<OUT>::run(acc[mi][ni][v]);
                        else *(LCMA_LDS float *)at = acc[mi][ni][v];
                    }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); // (for the compiler: the reads stay behind the writes)
#pragma unroll
                for (int it = 0; it < NIT; ++it) {
                    const int idx = it * 64 + s.lane, row = idx / CPRW, ch = idx % CPRW;
                    const u32x4 v = *(LCMA_LDS u32x4 *)(strip + row * PITCH + ch * 16);
                    const uint32_t colb = (uint32_t)(s.wn * WN) * OES + ch * 16; // byte column inside the tile
                    // a vector past N goes to the end of the extent and is dropped (N is a whole number of vectors); rows
                    // past M fall outside the extent by themselves
                    const uint32_t off = ((uint32_t)z * TN * OES + colb < p.n_row_b)
                                             ? c_base + (uint32_t)(s.wm * WM + mi * 32 + h * SR + row) * p.ldc_b + colb
                                             : p.c_bytes;
                    __builtin_amdgcn_raw_buffer_store_b128(v, s.rc, (int)off, 0, kStreamed);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
        }
        __syncthreads();
    }

    // fp32 partial sums of a piece, in accumulator order (value v of tile (mi, ni) of every thread): the fix-up kernel
    // reads them back in the same order, so no layout needs to be agreed on beyond this function and piece_value.
    static LCMA_DEV void store_piece(const PlaneGemmParams &p, const State &s, int slot, const f32x16 (&acc)[NMI][NNI]) {
        float *dst = (float *)p.partial + (int64_t)slot * TILE_FLOATS;
#pragma unroll
        for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NNI; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = {acc[mi][ni][4 * q], acc[mi][ni][4 * q + 1], acc[mi][ni][4 * q + 2], acc[mi][ni][4 * q + 3]};
                    *(f32x4 *)(dst + ((((mi * NNI + ni) * 4 + q) * NT) + threadIdx.x) * 4) = v;
                }
    }

    // Second kernel: one work-group per boundary between work-groups u - 1 and u.  If that boundary is the first one
    // inside its tile-product, the work-group adds the pieces of the tile-product in ascending work-group order (the
    // head piece of u - 1, then the pieces of u, u + 1, ... that start inside it), rounds once and stores the tile.
    static LCMA_DEV void fixup(const PlaneGemmParams &p, LCMA_LDS char *lds) {
        const int u = blockIdx.x + 1, ny = p.ny;
        const int64_t total = (int64_t)p.jobs * ny, b = (int64_t)u * p.cap;
        if (b >= total || b % ny == 0) return;            // no tile-product straddles this boundary
        const int job = (int)(b / ny);
        if (b - p.cap > (int64_t)job * ny) return;        // an earlier boundary lies inside the same tile-product
        State s;
        const int tid = threadIdx.x;
        s.lane = tid & 63;
        s.w = tid >> 6;
        s.wm = s.w / WGN;
        s.wn = s.w % WGN;
        s.l32 = s.lane & 31;
        s.lh = s.lane >> 5;
        s.rc = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)p.c_bytes, 0x00020000);
        f32x16 acc[NMI][NNI];
        auto add_piece = [&](int slot, bool first) {
            const float *src = (const float *)p.partial + (int64_t)slot * TILE_FLOATS;
#pragma unroll
            for (int mi = 0; mi < NMI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NNI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x4 v = *(const f32x4 *)(src + ((((mi * NNI + ni) * 4 + q) * NT) + threadIdx.x) * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[mi][ni][4 * q + e] = first ? v[e] : acc[mi][ni][4 * q + e] + v[e];
                    }
        };
        add_piece((u - 1) * 2 + 1, true);                 // the head piece (starts at step 0 of the tile-product)
        for (int v = u; (int64_t)v * p.cap < (int64_t)(job + 1) * ny && (int64_t)v * p.cap < total; ++v) add_piece(v * 2, false);
        const int tiles = p.nx * p.nz, plane = job / tiles;
        int id = job - plane * tiles;
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
        store_tile(p, s, lds, plane, x, z, acc);
    }
};

} // namespace lcma
