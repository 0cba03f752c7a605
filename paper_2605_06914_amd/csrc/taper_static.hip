// Device memory that belongs to no context and is never allocated: the scratch array behind
// taper_decode_step_attention_static (for callers that cannot allocate device memory).  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.
#include "taper_internal.h"

namespace taper {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code the array's name is only a handle for the symbol, not a device address: what kernels,
// copies and fills are given is the address looked up here, once per device.
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];

hipError_t static_scratch(int device, void** ptr) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // of the current device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return hipSuccess;
}

// Clears n 32-bit words (a kernel rather than a memset node: the call may be recorded into a graph).
__global__ __launch_bounds__(256) void zero_words_kernel(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_zero_words(int32_t* p, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

}  // namespace taper
