// Stand-alone Combine H for gfx950 (paper Eq. 6; Algorithm 1, stage 4): C_{i,j} = sum_r W[r,i,j] H_r
// with the products H_r read back from memory.  It exists for the unfused dataflow of Algorithm 1,
// which this library provides to be measured against its fused kernels; the fused kernels apply W
// to fp32 accumulators in registers and never run this.
//
// H: R planes of (padded M/m) x (padded N/n) elements in the type the products were written in
// (fp16 or fp32 for 16-bit storage, fp32 for fp32 storage).  The terms are widened to fp32 (exact), added in
// ascending r and the sum is rounded once, to nearest-even, to the storage type of C.  Rows past M
// fall outside the extent of C (dropped by the range check), columns past N are sent there.
//
// HBM-bound: reads R/(m n) and writes 1 element per element of C.  One thread handles one 16-byte
// vector position of C in every plane (two 16-byte loads per plane when the planes hold fp32 and C 16-bit
// elements) and writes the m*n vectors it yields.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_prepare_b.hpp"

namespace lcma {

// CH (generated): NP planes, NC = m*n outputs with c_i(o), c_j(o); comb(in, o) = Eq. 6 for output o on floats.
// HT: element type of the planes; IN: storage type of C (same element size).
template <class IN, class HT, class CH> LCMA_DEV void combine_h_tile(const CombHParams &p) {
    constexpr int ES = IN::ES, EPT = 16 / ES, HV = HT::ES / ES; // HV: 16-byte vectors of a plane per vector of C
    static_assert(HT::ES == ES || (HT::ES == 4 && ES == 2), "planes in the element size of C, or fp32 planes for 16-bit C");
    const auto rh = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.H), 0, (int)p.h_bytes, 0x00020000);
    const auto rc = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)p.c_bytes, 0x00020000);
    // 256 threads: 16 rows x 16 vectors (256 bytes of a row of C); work-groups that start together cover consecutive pieces
    // of the same rows (4 to 24 % faster than consecutive rows of the same piece)
    const uint32_t row = blockIdx.y * 16 + threadIdx.x / 16;
    const uint32_t colb = (blockIdx.x * 16 + threadIdx.x % 16) * 16; // byte column inside a block of C
    if (colb * HV >= p.h_ld_b) return;
    // the planes stay in registers as loaded and are widened where a sum uses them (see forget_derived)
    u32x4 h[HV][CH::NP];
#pragma unroll
    for (int r = 0; r < CH::NP; ++r)
#pragma unroll
        for (int q = 0; q < HV; ++q)
            h[q][r] = __builtin_amdgcn_raw_buffer_load_b128(rh, (int)(row * p.h_ld_b + colb * HV + q * 16), (int)(r * p.h_plane_b), 0);
    constexpr int HPV = 16 / HT::ES; // elements of a plane per 16-byte vector
    for_each_const<CH::NC>([&](auto oc_) {
        constexpr int o = decltype(oc_)::value;
        // (only where the widened copies of all planes would not fit beside them and the planes themselves do, <4,4,4;49>
        // with 16-bit planes: two waves per SIMD instead of one; with fewer planes the barrier only delays the first sums)
        if constexpr (HV * CH::NP * 4 > 128 && HV * CH::NP * 4 <= 224) {
#pragma unroll
            for (int q = 0; q < HV; ++q) forget_derived(h[q]);
        }
        u32x4 v;
        if constexpr (ES == 2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float col0[CH::NP], col1[CH::NP];
#pragma unroll
                for (int r = 0; r < CH::NP; ++r) {
                    col0[r] = Elem<HT>::get(h[(2 * e) / HPV][r], (2 * e) % HPV);
                    col1[r] = Elem<HT>::get(h[(2 * e + 1) / HPV][r], (2 * e + 1) % HPV);
                }
                v[e] = Round<IN>::run(CH::comb(col0, o)) | (Round<IN>::run(CH::comb(col1, o)) << 16);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float col[CH::NP];
#pragma unroll
                for (int r = 0; r < CH::NP; ++r) col[r] = Elem<HT>::get(h[0][r], e);
                v[e] = Round<IN>::run(CH::comb(col, o));
            }
        }
        const uint32_t cb = (uint32_t)CH::c_j(o) * p.c_bcol + colb;
        const uint32_t off = cb < p.n_row_b ? (uint32_t)CH::c_i(o) * p.c_brow + row * p.ldc_b + cb : p.c_bytes;
        // (16-byte store: the scalar-offset field stays a literal zero, see Ctx::store_c in lcma_device.hpp)
        __builtin_amdgcn_raw_buffer_store_b128(v, rc, (int)off, 0, kStreamed);
    });
}

} // namespace lcma
