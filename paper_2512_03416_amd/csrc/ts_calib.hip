// Bandwidth calibration kernels: a plain streaming copy and a streaming read of known size.
// They give the HBM counters and the achievable-bandwidth figure a fixed point to be scaled
// against; they are not part of the attention pass.
#include <hip/hip_runtime.h>

#include "tokenscale.h"

namespace {

__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void calib_read_kernel(const uint4* __restrict__ src, unsigned* result, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    unsigned acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) *result = acc;      // practically never taken: keeps the loads alive
}

}  // namespace

extern "C" int ts_calib_copy(void* stream, const void* src, void* dst, int64_t bytes)
{
    if (!src || !dst || bytes <= 0 || bytes % 16) return TS_ERR_INVALID_ARG;
    hipLaunchKernelGGL(calib_copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                       (uint4*)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? TS_OK : TS_ERR_HIP;
}

extern "C" int ts_calib_read(void* stream, const void* src, void* result4, int64_t bytes)
{
    if (!src || !result4 || bytes <= 0 || bytes % 16) return TS_ERR_INVALID_ARG;
    hipLaunchKernelGGL(calib_read_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                       (unsigned*)result4, bytes / 16);
    return hipGetLastError() == hipSuccess ? TS_OK : TS_ERR_HIP;
}
