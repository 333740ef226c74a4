// Measurement probes for bench.py, built into their own library (libpatdnn_probes.so):
// nothing of the method is computed here.
//   patdnn_probe_copy  a plain device-to-device copy of known size.  Timed, it gives the
//                      achievable HBM stream rate; profiled beside the convolution kernels,
//                      its FETCH_SIZE / WRITE_SIZE readings for a known byte count give the
//                      factor that turns the same counters of the other kernels into bytes.
//   patdnn_probe_fma   independent fp32 FMA chains in registers: the achievable rate of the
//                      plain (non-packed) vector FMA that the convolution kernels use.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/patdnn_probes.h"

namespace {

__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

constexpr int kChains = 24;

__global__ __launch_bounds__(256) void fma_probe_kernel(float* out, int iters, float a, float b)
{
    float acc[kChains];
#pragma unroll
    for (int k = 0; k < kChains; ++k) acc[k] = (float)(threadIdx.x + k);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < kChains; ++k) acc[k] = fmaf(acc[k], a, b);
    }
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < kChains; ++k) s += acc[k];
    if (s == 123.456f) out[0] = s;                   // keeps the chains alive; never true in practice
}

}  // namespace

extern "C" int32_t patdnn_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) return 1;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 256 * 64 ? (n16 + 255) / 256 : 256 * 64);
    hipLaunchKernelGGL(copy_probe_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

extern "C" int32_t patdnn_probe_fma(float* out, int32_t blocks, int32_t iters, void* stream, double* flops)
{
    if (!out || blocks <= 0 || iters <= 0) return 1;
    hipLaunchKernelGGL(fma_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       out, iters, 0.999f, 0.001f);
    if (flops) *flops = 2.0 * kChains * 256.0 * (double)blocks * (double)iters;
    return hipGetLastError() == hipSuccess ? 0 : 4;
}
