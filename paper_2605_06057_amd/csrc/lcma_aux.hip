// Hand-written auxiliary kernels of the LCMA library for gfx950 (everything that is not generated per scheme).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lcma_device.hpp"
#include "lcma_prepare_b.hpp"

namespace {
using namespace lcma;

// C = beta * C on an M x N matrix: what Eq. 1 leaves of C = alpha * A B + beta * C when K = 0.  One thread per
// 16-byte vector; beta == 0 writes zeros without reading C (so NaN in the old contents does not survive).
template <class IN>
__global__ __launch_bounds__(256) void scale_c(char *C, int64_t rows, uint32_t row_bytes, int64_t ld_bytes, float beta) {
    const uint32_t vec = blockIdx.x * 256 + threadIdx.x; // vector inside the row
    const int64_t row = blockIdx.y;
    if (vec * 16 >= row_bytes || row >= rows) return;
    u32x4 *ptr = (u32x4 *)(C + row * ld_bytes + (int64_t)vec * 16);
    u32x4 out = {0u, 0u, 0u, 0u};
    if (beta != 0.f) {
        constexpr int EPT = 16 / IN::ES;
        float v[EPT];
        Widen<IN>::run(*ptr, v);
        if constexpr (IN::ES == 2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = Round<IN>::run(beta * v[2 * e]) | (Round<IN>::run(beta * v[2 * e + 1]) << 16);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = Round<IN>::run(beta * v[e]);
        }
    }
    *ptr = out;
}
// Range guard for bf16 storage (the LCMA kernels form and multiply their combinations in fp16): bit 0 of *flags is set
// when some magnitude exceeds 32752 (half the largest fp16 value: a two-term sum may overflow; beyond 65504 the
// conversion itself saturates), bit 1 when some non-zero magnitude is below 2^-14 (fp16 subnormal range: low bits of
// the 8-bit significand are dropped).  One 16-byte vector per thread and iteration; one atomic OR per wave that found
// something.
__global__ __launch_bounds__(256) void range_flags_bf16(const char *X, int64_t rows, uint32_t row_bytes, int64_t ld_bytes, uint32_t *flags) {
    uint32_t found = 0;
    const int64_t vecs_per_row = row_bytes / 16, total = rows * vecs_per_row;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        const int64_t row = v / vecs_per_row, c = v - row * vecs_per_row;
        const u32x4 raw = *(const u32x4 *)(X + row * ld_bytes + c * 16);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t mag = (h ? raw[e] >> 16 : raw[e] & 0xffffu) & 0x7fffu; // bf16 magnitude bits
                if (mag > 0x46ffu) found |= 1u;              // > 32752 (0x46FF is 32640, the largest bf16 not above 32752), Inf, NaN
                if (mag != 0 && mag < 0x3880u) found |= 2u;  // < 2^-14 (0x3880)
            }
    }
    if (found) atomicOr(flags, found);
}
__global__ void zero_word(uint32_t *w) { *w = 0; }
// Measurement aid: what the matrix pipe sustains with no memory traffic at all.  Every wave takes eight fragments from
// `src` (4096 vectors of eight fp16 values) and runs `iters` rounds of eight independent 32x32x16 fp16 instructions on them
// (eight accumulator tiles, two waves per SIMD: the pipe is never waiting for a result).  On MI355X the rate depends on the
// VALUES: the chip runs into its power limit on operands that toggle many bits.
__global__ __launch_bounds__(256, 2) void mfma_probe(const f16x8 *src, float *sink, int iters) {
    f16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = src[(threadIdx.x + 256 * i) & 4095];
        b[i] = src[(threadIdx.x * 7 + 64 * i + 13) & 4095];
    }
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) zero(acc[i]);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i & 3], b[(i >> 1) & 3], acc[i], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += acc[i][e];
    sink[blockIdx.x * 256 + threadIdx.x] = sum; // (keeps the loop alive)
}
} // namespace

// 2048 work-groups of 256 threads; src: 64 KiB, sink: 2 MiB
extern "C" int lcma_launch_mfma_probe(const void *src, void *sink, int iters, void *stream) {
    mfma_probe<<<dim3(2048), dim3(256), 0, (hipStream_t)stream>>>((const f16x8 *)src, (float *)sink, iters);
    return (int)hipGetLastError();
}

extern "C" int lcma_launch_range_flags_bf16(const void *X, int64_t rows, int64_t row_bytes, int64_t ld_bytes, void *flags, void *stream) {
    const hipStream_t st = (hipStream_t)stream;
    zero_word<<<1, 1, 0, st>>>((uint32_t *)flags);
    const int64_t total = rows * (row_bytes / 16);
    if (total == 0) return (int)hipGetLastError();
    int64_t grid = (total + 255) / 256;
    if (grid > 4096) grid = 4096;
    range_flags_bf16<<<dim3((unsigned)grid), dim3(256), 0, st>>>((const char *)X, rows, (uint32_t)row_bytes, ld_bytes, (uint32_t *)flags);
    return (int)hipGetLastError();
}

extern "C" int lcma_launch_scale_c(void *C, int64_t rows, int64_t row_bytes, int64_t ld_bytes, int dtype, float beta,
                                   void *stream) {
    const hipStream_t st = (hipStream_t)stream;
    for (int64_t r0 = 0; r0 < rows; r0 += 65535) { // grid.y is limited to 65535
        const int64_t nr = rows - r0 < 65535 ? rows - r0 : 65535;
        const dim3 grid((unsigned)((row_bytes / 16 + 255) / 256), (unsigned)nr), block(256);
        char *base = (char *)C + r0 * ld_bytes;
        if (dtype == 0) scale_c<F32><<<grid, block, 0, st>>>(base, nr, (uint32_t)row_bytes, ld_bytes, beta);
        else if (dtype == 1) scale_c<BF16><<<grid, block, 0, st>>>(base, nr, (uint32_t)row_bytes, ld_bytes, beta);
        else scale_c<F16><<<grid, block, 0, st>>>(base, nr, (uint32_t)row_bytes, ld_bytes, beta);
        if (const hipError_t e = hipGetLastError()) return (int)e;
    }
    return 0;
}
