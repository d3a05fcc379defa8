// dwm_conv_forward_static: the forward convolution for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// It is dwm_conv_forward with the plan's workspace -- the transformed input V, the partial
// outputs and the arrival counters of the contraction's split tiles -- replaced by a
// file-scope device array of fixed size that lives in the library's code object.
#include <hip/hip_runtime.h>

#include <mutex>

#include "plan.hpp"

namespace {

constexpr size_t kScratchBytes = DWM_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// One copy per GPU the code object is loaded on; zero-initialised, kept until the process ends.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle for the symbol: the device address is asked for
// once per device, with that device current, and kept.
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];

dwm_status_t scratch_of_current_device(float** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DWM_ERR_HIP;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DWM_ERR_HIP;
        if (reinterpret_cast<uintptr_t>(ptr) & 255u) return DWM_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<float*>(g_scratch_ptr[dev]);
    return DWM_OK;
}

}  // namespace

extern "C" {

size_t dwm_static_scratch_bytes(void) { return kScratchBytes; }

dwm_status_t dwm_conv_forward_static(const dwm_plan_t* plan, const float* x_dev, const float* Ugw_dev, float* y_dev,
                                     void* stream)
{
    if (!plan || !x_dev || !Ugw_dev || !y_dev) return DWM_ERR_INVALID_ARG;
    // the single-kernel path keeps V in registers and has no scratch at all
    if (plan->use_fused()) return dwm::launch_fused_forward(*plan, x_dev, Ugw_dev, y_dev, stream);
    if (plan->ws_need_bytes() > kScratchBytes) return DWM_ERR_WORKSPACE;
    float* ws = nullptr;
    dwm_status_t st = scratch_of_current_device(&ws);
    if (st != DWM_OK) return st;
    // the input transform writes every element of V that the contraction reads and clears the
    // arrival counters, so nothing of the previous call's contents survives into this one
    st = dwm::launch_input_transform(*plan, x_dev, ws, stream);
    if (st != DWM_OK) return st;
    return dwm::launch_contract_output(*plan, Ugw_dev, ws, y_dev, stream);
}

}  // extern "C"
