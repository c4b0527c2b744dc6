// Element-wise kernels of the DENSE baseline step that the benchmark times next to the sparse one (measurement aid,
// not part of the method): eq. (2) y2 = max(y1, 0)^2 and eq. (6) dy1 = 2 * dy2 * max(y1, 0) of Section 2.1 on whole
// [T, F] tensors, each in ONE pass over HBM (16 bytes per lane, grid-stride), so that the dense step the speed-up is
// quoted against pays what a fused framework kernel would pay and not one pass per primitive op.
#include "../../include/sparseffn.h"
#include "common.hpp"

namespace sffn {

__device__ __forceinline__ uint32_t sq2(uint32_t w) {            // two bf16 -> max(.,0)^2, one RNE each
    const float a = bf2f(w & 0xFFFFu), b = bf2f(w >> 16);
    const float ra = a > 0.0f ? a : 0.0f, rb = b > 0.0f ? b : 0.0f;
    return f2bf2(ra * ra, rb * rb);
}
__device__ __forceinline__ uint32_t dsq2(uint32_t d, uint32_t y) {
    const float ya = bf2f(y & 0xFFFFu), yb = bf2f(y >> 16);
    return f2bf2(2.0f * bf2f(d & 0xFFFFu) * (ya > 0.0f ? ya : 0.0f), 2.0f * bf2f(d >> 16) * (yb > 0.0f ? yb : 0.0f));
}

__global__ void __launch_bounds__(256) dense_sqrelu_kernel(const uint4* __restrict__ y1, uint4* __restrict__ y2, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) {
        const uint4 v = y1[i];
        y2[i] = make_uint4(sq2(v.x), sq2(v.y), sq2(v.z), sq2(v.w));
    }
}

__global__ void __launch_bounds__(256) dense_dsqrelu_kernel(const uint4* __restrict__ dy2, const uint4* __restrict__ y1,
                                                           uint4* __restrict__ dy1, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) {
        const uint4 d = dy2[i], y = y1[i];
        dy1[i] = make_uint4(dsq2(d.x, y.x), dsq2(d.y, y.y), dsq2(d.z, y.z), dsq2(d.w, y.w));
    }
}

static unsigned grid_for(int64_t n16) {
    const int64_t blocks = (n16 + 255) / 256;
    return (unsigned)(blocks < 256 * 32 ? blocks : 256 * 32);      // at most 32 workgroups per CU, grid-stride beyond
}

}  // namespace sffn

extern "C" {

int sffn_dense_sqrelu(const uint16_t* y1, uint16_t* y2, int64_t n, void* stream) {
    if (!y1 || !y2 || n <= 0 || n % 8 != 0 || ((uintptr_t)y1 & 15) || ((uintptr_t)y2 & 15)) return SFFN_EINVAL;
    hipLaunchKernelGGL(sffn::dense_sqrelu_kernel, dim3(sffn::grid_for(n / 8)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4*)y1, (uint4*)y2, n / 8);
    return hipGetLastError() == hipSuccess ? SFFN_OK : SFFN_EHIP;
}

int sffn_dense_dsqrelu(const uint16_t* dy2, const uint16_t* y1, uint16_t* dy1, int64_t n, void* stream) {
    if (!dy2 || !y1 || !dy1 || n <= 0 || n % 8 != 0 || ((uintptr_t)dy2 & 15) || ((uintptr_t)y1 & 15) || ((uintptr_t)dy1 & 15)) return SFFN_EINVAL;
    hipLaunchKernelGGL(sffn::dense_dsqrelu_kernel, dim3(sffn::grid_for(n / 8)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4*)dy2, (const uint4*)y1, (uint4*)dy1, n / 8);
    return hipGetLastError() == hipSuccess ? SFFN_OK : SFFN_EHIP;
}

}  // extern "C"
