// lcma_gemm_unfused_static: the unfused dataflows (Algorithm 1 / Algorithm 2 as printed) for callers that cannot
// allocate device memory or hand over a workspace: code under HIP graph capture, tight serving loops, harnesses
// that forbid hipMalloc.  The planes At_r, Bt_r and H_r live in a file-scope device array instead of a
// caller-provided workspace.  Nothing here allocates: no hipMalloc / hipFree, no allocating library call.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "host_common.h"

#define LCMA_STATIC_SCRATCH_BYTES (32u << 20)

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: kernels get the device address kept in g_scratch below.
static __device__ __align__(256) unsigned char scratch[LCMA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch[kMaxDevices];              // device address of `scratch` on each GPU, looked up once per device
std::atomic<int> g_state[kMaxDevices];     // 0 not looked up, 1 ready
std::mutex g_mu;

// Device address of this GPU's copy of the array (the device must be current), or nullptr with *err set.
void *scratch_of_current_device(int *err) {
    int dev = -1;
    if (const hipError_t e = hipGetDevice(&dev)) {
        *err = (int)e;
        return nullptr;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        *err = (int)hipErrorInvalidDevice;
        return nullptr;
    }
    if (g_state[dev].load(std::memory_order_acquire) == 0) {
        std::lock_guard<std::mutex> lock(g_mu);
        if (g_state[dev].load(std::memory_order_relaxed) == 0) {
            void *ptr = nullptr;
            if (const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) {
                *err = (int)e;
                return nullptr;
            }
            g_scratch[dev] = ptr;
            g_state[dev].store(1, std::memory_order_release);
        }
    }
    return g_scratch[dev];
}
} // namespace

extern "C" int64_t lcma_static_scratch_bytes(void) { return (int64_t)LCMA_STATIC_SCRATCH_BYTES; }

extern "C" lcma_status lcma_gemm_unfused_static(int level, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                                                const void *B, int64_t ldb, void *C, int64_t ldc, lcma_dtype dtype,
                                                const lcma_scheme *scheme, int reuse_bt, void *stream) {
    const char *who = "lcma_gemm_unfused_static";
    const int64_t need = lcma_unfused_workspace_bytes(M, N, K, dtype, scheme);
    if (need > (int64_t)LCMA_STATIC_SCRATCH_BYTES)
        return lcma::fail(LCMA_ERR_SHAPE, "%s: the planes of this shape take %lld bytes, the static buffer holds %lld; use "
                          "lcma_gemm_unfused with a workspace", who, (long long)need, (long long)LCMA_STATIC_SCRATCH_BYTES);
    int err = 0;
    void *ws = scratch_of_current_device(&err);
    if (!ws) return lcma::fail(LCMA_ERR_HIP, "%s: the address of the static buffer is not available (HIP error %d)", who, err);
    // every plane the kernels read is written first by the Combine stages of this call (zero padding included), so
    // nothing needs clearing; with reuse_bt the Bt planes of the previous call on this GPU are read as they are
    return lcma::gemm_unfused(who, level, M, N, K, A, lda, B, ldb, C, ldc, dtype, scheme, ws,
                              (int64_t)LCMA_STATIC_SCRATCH_BYTES, reuse_bt, stream);
}
