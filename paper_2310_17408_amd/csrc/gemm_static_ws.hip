// gemm_ex_static_ws: gemm_ex for callers that cannot allocate device memory.  The partial tiles of a split
// K loop, which gemm_ex keeps in the caller's workspace, live here in an array that is part of the
// library's code object; every GPU the library runs on holds its own copy at its own address until the
// process ends.  Nothing in this file allocates or frees.
#include "../../include/mi_gemm.h"

#include <hip/hip_runtime.h>

#include <atomic>

// Only host code names the array (scratch_address below); that use is what makes the compiler keep it in
// the device code object and give it a symbol the runtime can look up.
static __device__ __align__(256) unsigned char scratch[MI_GEMM_STATIC_WS_BYTES];

namespace {

// Device address of `scratch` on each GPU, looked up once per device.  In host code the array's name
// is only a handle for hipGetSymbolAddress; kernels get the looked-up address.
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// 0 and the address in *ptr, or the HIP error of the lookup
int scratch_address(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // the current device's copy
        if (e != hipSuccess) return (int)e;
        if (p == nullptr) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same value
    }
    *ptr = p;
    return 0;
}

}  // namespace

extern "C" int gemm_ex_static_ws(int dtype, int layout, int transa, int transb, int64_t M, int64_t N, int64_t K,
                                 const void *alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                                 const void *beta, void *C, int64_t ldc, void *stream)
{
    // what gemm_ex would be given by a caller who sizes the workspace with gemm_workspace_bytes; 0 for
    // sizes gemm_ex rejects (it then reports which) and for problems that never split
    const size_t need = gemm_workspace_bytes(dtype, M, N, K);
    if (need > (size_t)MI_GEMM_STATIC_WS_BYTES) return MI_GEMM_STATUS_STATIC_WS_TOO_SMALL;
    void *ws = nullptr;
    if (need > 0) {
        const int rc = scratch_address(&ws);
        if (rc != 0) return rc;
    }
    return gemm_ex(dtype, layout, transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, ws, need, stream);
}
