// ffn_sparse_step for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc): the step's workspace is a file-scope device array of this library instead of a caller buffer.
// Every GPU the library runs on holds its own copy of the array (at its own address) until the process ends.
#include <mutex>
#include <stdio.h>

#include "../../include/sparseffn.h"
#include <hip/hip_runtime.h>

namespace {

// The workspace itself.  In host code this name is only a stand-in for the device symbol: its device address is obtained
// once per device with hipGetSymbolAddress (below) and only that address is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[SFFN_NOALLOC_WORKSPACE_MAX];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};     // device address of `scratch` on device d, filled on the first call there
std::mutex g_mu;

}  // namespace

extern "C" int sffn_noalloc_set_error(int code, const char* text);   // api.hip: records the text behind sffn_last_error()

extern "C" int ffn_sparse_step_noalloc(const sffn_cfg* cfg, const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1,
                                       const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* stream) {
    // size check first: no HIP call has been made when a request is refused
    const size_t need = sffn_workspace_bytes(cfg);
    if (need == 0)
        return sffn_noalloc_set_error(SFFN_EINVAL, "ffn_sparse_step_noalloc: T, D, F must be positive multiples of 64, V = 64, M in {8, 16, 32, 64}, F a multiple of 2 M");
    if (need > (size_t)SFFN_NOALLOC_WORKSPACE_MAX) {
        char msg[200];
        snprintf(msg, sizeof(msg), "ffn_sparse_step_noalloc: this shape needs %zu bytes of workspace, the built-in buffer holds %zu; use ffn_sparse_step",
                 need, (size_t)SFFN_NOALLOC_WORKSPACE_MAX);
        return sffn_noalloc_set_error(SFFN_EWORKSPACE, msg);
    }
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return sffn_noalloc_set_error(SFFN_EHIP, e != hipSuccess ? hipGetErrorString(e) : "ffn_sparse_step_noalloc: device index out of range");
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (g_scratch_ptr[dev] == nullptr) {        // once per device, with that device current
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || p == nullptr)
                return sffn_noalloc_set_error(SFFN_EHIP, e != hipSuccess ? hipGetErrorString(e) : "ffn_sparse_step_noalloc: no device address for the built-in workspace");
            g_scratch_ptr[dev] = p;
        }
        ws = g_scratch_ptr[dev];
    }
    // Same kernels, same launch order as ffn_sparse_step; every region of the workspace that a kernel reads is written earlier
    // in the same call, so contents left by a previous (larger or smaller) call are never seen and nothing has to be cleared.
    return ffn_sparse_step(cfg, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, ws, need, stream);
}
