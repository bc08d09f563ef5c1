// lqer_linear_forward_static: the forward pass for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid it).  Same kernels as lqer_linear_forward; what that
// call takes as a caller-owned workspace (the quantized activations, the partial sums of T, the tiled kernel's
// flag words) lives here in one file-scope device array that every GPU the library runs on holds until the
// process ends.
#include <mutex>

#include "lqer_internal.h"

namespace {

constexpr size_t kScratchBytes = (size_t)32 << 20;       // 32 MiB per device

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a stand-in for the symbol, not a device address: the address of each device's copy
// is looked up once per device, with that device current, and only that pointer is ever handed to kernels.
constexpr int kMaxDevices = 64;
std::once_flag g_once[kMaxDevices];
void* g_ptr[kMaxDevices];
hipError_t g_err[kMaxDevices];

hipError_t scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::call_once(g_once[dev], [dev] {
        void* p = nullptr;
        g_err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        g_ptr[dev] = (g_err[dev] == hipSuccess) ? p : nullptr;
    });
    if (g_err[dev] != hipSuccess) return g_err[dev];
    if (g_ptr[dev] == nullptr) return hipErrorInvalidSymbol;
    *out = g_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int lqer_linear_forward_static(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx,
                                          float* Y_dev, int64_t ldy, void* hip_stream) {
    if (!layer) return LQER_ERR_NULL;
    void* ws = nullptr;
    if (scratch_of_current_device(&ws) != hipSuccess) return LQER_ERR_HIP;
    return lqer::forward_in_scratch(layer, X_dev, M, ldx, Y_dev, ldy, ws, kScratchBytes, hip_stream);
}
