// Scheme-independent quantisation kernel of the FP8 path.
#include "lcma_fp8.hpp"

using namespace lcma;

extern "C" __global__ __launch_bounds__(256) void lcma_k_fp8_quantize_rows(const lcma::Fp8QuantParams p) {
    fp8_quantize_rows_tile(p);
}

extern "C" int lcma_launch_fp8_quantize_rows(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream) {
    lcma_k_fp8_quantize_rows<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);
    return (int)hipGetLastError();
}
