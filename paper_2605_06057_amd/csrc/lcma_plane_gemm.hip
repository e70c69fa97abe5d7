// Instances of the plane GEMM (csrc/lcma_plane_gemm.hpp) and of its fix-up kernel.
#include "lcma_plane_gemm.hpp"

using namespace lcma;

#define LCMA_PLANE_GEMM(NAME, KIND, TM, TN, WGM, WGN, OCC, OUT)                                                        \
    extern "C" __global__ __launch_bounds__(64 * WGM * WGN, OCC) void lcma_k_pg_##NAME(const lcma::PlaneGemmParams p) { \
        using G = PlaneGemm<KIND, TM, TN, WGM, WGN, OUT, false>;                                                       \
        __shared__ __attribute__((aligned(16))) char smem[G::LDS_BYTES];                                               \
        G::run(p, (LCMA_LDS char *)smem);                                                                              \
    }                                                                                                                  \
    extern "C" __global__ __launch_bounds__(64 * WGM * WGN, OCC) void lcma_k_pg_split_##NAME(const lcma::PlaneGemmParams p) { \
        using G = PlaneGemm<KIND, TM, TN, WGM, WGN, OUT, true>;                                                        \
        __shared__ __attribute__((aligned(16))) char smem[G::LDS_BYTES];                                               \
        G::run(p, (LCMA_LDS char *)smem);                                                                              \
    }                                                                                                                  \
    extern "C" __global__ __launch_bounds__(64 * WGM * WGN) void lcma_k_pg_fixup_##NAME(const lcma::PlaneGemmParams p) { \
        using G = PlaneGemm<KIND, TM, TN, WGM, WGN, OUT, true>;                                                        \
        __shared__ __attribute__((aligned(16))) char smem[G::LDS_BYTES];                                               \
        G::fixup(p, (LCMA_LDS char *)smem);                                                                            \
    }                                                                                                                  \
    /* one tile-product per work-group when cap is a whole tile-product and there are as many work-groups as              \
       tile-products, else the persistent kernel and the kernel that adds the pieces */                                  \
    extern "C" int lcma_launch_pg_##NAME(const lcma::PlaneGemmParams *p, void *stream) {                               \
        if (p->cap == p->ny && p->units == p->jobs) {                                                                  \
            lcma_k_pg_##NAME<<<dim3(p->units), dim3(64 * WGM * WGN), 0, (hipStream_t)stream>>>(*p);                    \
            return (int)hipGetLastError();                                                                             \
        }                                                                                                              \
        lcma_k_pg_split_##NAME<<<dim3(p->units), dim3(64 * WGM * WGN), 0, (hipStream_t)stream>>>(*p);                  \
        if (const hipError_t e = hipGetLastError()) return (int)e;                                                     \
        if (p->cap % p->ny && p->units > 1)                                                                            \
            lcma_k_pg_fixup_##NAME<<<dim3(p->units - 1), dim3(64 * WGM * WGN), 0, (hipStream_t)stream>>>(*p);          \
        return (int)hipGetLastError();                                                                                 \
    }

// name: operand kind, tile, type of C
LCMA_PLANE_GEMM(fp8_t256_bf16, FP8, 256, 256, 2, 4, 1, BF16)
LCMA_PLANE_GEMM(fp8_t128_bf16, FP8, 128, 128, 2, 2, 2, BF16)
LCMA_PLANE_GEMM(fp8_t256_f16, FP8, 256, 256, 2, 4, 1, F16)
LCMA_PLANE_GEMM(fp8_t128_f16, FP8, 128, 128, 2, 2, 2, F16)
LCMA_PLANE_GEMM(f16_t256_f16, F16, 256, 256, 2, 4, 1, F16)
LCMA_PLANE_GEMM(f16_t128_f16, F16, 128, 128, 2, 2, 2, F16)
LCMA_PLANE_GEMM(f16_t256_f32, F16, 256, 256, 2, 4, 1, F32)
LCMA_PLANE_GEMM(f16_t128_f32, F16, 128, 128, 2, 2, 2, F32)
LCMA_PLANE_GEMM(bf16_t256_bf16, BF16, 256, 256, 2, 4, 1, BF16)
LCMA_PLANE_GEMM(bf16_t128_bf16, BF16, 128, 128, 2, 2, 2, BF16)


