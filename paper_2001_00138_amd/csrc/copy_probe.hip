// A plain device-to-device copy of known size.  It computes nothing of the method: it
// is the yardstick for hardware traffic counters - profiled next to the convolution
// kernels, its FETCH_SIZE / WRITE_SIZE readings for a known byte count give the factor
// that turns the same counters of the other kernels into bytes.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/patdnn.h"

namespace patdnn {

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace patdnn

extern "C" patdnn_status_t patdnn_copy_probe(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0)
        return PATDNN_EINVAL;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 256 * 64 ? (n16 + 255) / 256 : 256 * 64);
    hipLaunchKernelGGL(patdnn::copy_probe_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
    return hipGetLastError() == hipSuccess ? PATDNN_OK : PATDNN_EHIP;
}
