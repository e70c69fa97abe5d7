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
} // namespace

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
