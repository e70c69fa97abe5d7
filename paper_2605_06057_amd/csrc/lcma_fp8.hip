// Scheme-independent kernels of the FP8 path: row quantisation and the block-scaled GEMM on E4M3 codes.
#include "lcma_fp8.hpp"

using namespace lcma;

extern "C" __global__ __launch_bounds__(256) void lcma_k_fp8_quantize_rows(const lcma::Fp8QuantParams p) {
    fp8_quantize_rows_tile(p);
}

extern "C" int lcma_launch_fp8_quantize_rows(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream) {
    lcma_k_fp8_quantize_rows<<<dim3(gx, gy), dim3(256), 0, (hipStream_t)stream>>>(*p);
    return (int)hipGetLastError();
}

#define LCMA_FP8_GEMM(NAME, TM, TN, WGM, WGN, OCC, BATCH, OUT)                                                       \
    extern "C" __global__ __launch_bounds__(64 * WGM * WGN, OCC) void lcma_k_fp8_gemm_##NAME(const lcma::Fp8GemmParams p) { \
        using G = Fp8Gemm<TM, TN, WGM, WGN, BATCH, OUT>;                                                              \
        __shared__ __attribute__((aligned(16))) char smem[G::LDS_BYTES];                                              \
        G::run(p, (LCMA_LDS char *)smem);                                                                             \
    }                                                                                                                 \
    extern "C" int lcma_launch_fp8_gemm_##NAME(const lcma::Fp8GemmParams *p, int grid, void *stream) {                \
        lcma_k_fp8_gemm_##NAME<<<dim3(grid), dim3(64 * WGM * WGN), 0, (hipStream_t)stream>>>(*p);                     \
        return (int)hipGetLastError();                                                                                \
    }

// C in bf16 (the plain workflow)
LCMA_FP8_GEMM(t256x256_bf16, 256, 256, 2, 4, 1, false, BF16)
LCMA_FP8_GEMM(t128x128_bf16, 128, 128, 2, 2, 2, false, BF16)
// batched over the R planes of a scheme, products stored in fp16 (stage 3 of Algorithm 1)
LCMA_FP8_GEMM(t256x256_f16g, 256, 256, 2, 4, 1, true, F16)
LCMA_FP8_GEMM(t128x128_f16g, 128, 128, 2, 2, 2, true, F16)
