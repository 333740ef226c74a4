// Variant 0: the reordered layer executed straight from the FKW arrays
// (paper section 5.2, the reorder-only code: filter -> pattern -> kernels of that
// pattern, no branches inside the kernel loop).  One lane per output pixel, one
// workgroup row per stored filter.  Handles every stride / pad / depthwise / dense
// case; it is the fallback for shapes the tiled variants do not cover.
// With T = __half the arrays hold binary16 values (weights, input, output) and the
// arithmetic stays fp32: the half-precision storage of the paper's GPU runs (section 6.1).
#include <hip/hip_fp16.h>

#include <type_traits>

#include "kernels.hpp"

namespace patdnn {

__device__ __forceinline__ float fkw_ld(const float* p) { return *p; }
__device__ __forceinline__ float fkw_ld(const __half* p) { return __half2float(*p); }
__device__ __forceinline__ void fkw_st(float* p, float v) { *p = v; }
__device__ __forceinline__ void fkw_st(__half* p, float v) { *p = __float2half_rn(v); }

template <class T>
struct FkwArgs {
    const int32_t* offset;
    const int32_t* reorder;
    const int32_t* index;
    const int32_t* stride;
    const T* weight;
    const uint16_t* masks;
    const T* in;
    const float* bias;
    T* out;
    int32_t num_patterns;
    int32_t n, c_in, c_out, h, w, ho, wo, conv_stride, pad, relu, pool;
};

template <int TAPS, class T>
__global__ __launch_bounds__(256) void fkw_conv_kernel(FkwArgs<T> a)
{
    const int s = blockIdx.y;                       // stored filter
    const int pix = blockIdx.x * 256 + threadIdx.x;
    const bool live = pix < a.ho * a.wo;
    const int oh = live ? pix / a.wo : 0;
    const int ow = live ? pix - oh * a.wo : 0;
    const int co = a.reorder[s];
    const int32_t kbase = a.offset[s];
    const int32_t* st = a.stride + (size_t)s * (a.num_patterns + 1);
    const size_t plane = (size_t)a.h * a.w;

    for (int img = blockIdx.z; img < a.n; img += gridDim.z) {
        const T* in_img = a.in + (size_t)img * a.c_in * plane;
        float acc = 0.0f;
        for (int p = 0; p < a.num_patterns; ++p) {
            const int32_t kb = kbase + st[p], ke = kbase + st[p + 1];
            if (kb == ke) continue;
            // the pattern's tap geometry for this lane, fixed for all its kernels
            unsigned m = a.masks[p];
            int rel[TAPS];
            bool ok[TAPS];
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int pos = __builtin_ctz(m);
                m &= m - 1;
                const int kh = pos / 3, kw = pos - 3 * kh;
                const int ih = oh * a.conv_stride + kh - a.pad;
                const int iw = ow * a.conv_stride + kw - a.pad;
                ok[t] = live && ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
                rel[t] = ok[t] ? ih * a.w + iw : 0;
            }
            for (int32_t k = kb; k < ke; ++k) {
                const T* src = in_img + (size_t)a.index[k] * plane;
                const T* wk = a.weight + (size_t)k * TAPS;
#pragma unroll
                for (int t = 0; t < TAPS; ++t) {
                    const float x = ok[t] ? fkw_ld(src + rel[t]) : 0.0f;
                    acc = fmaf(fkw_ld(wk + t), x, acc);
                }
            }
        }
        if (a.bias) acc += a.bias[co];
        if constexpr (std::is_same<T, float>::value) {
            if (a.pool) {
                // ReLU + 2x2 max pooling folded into the (zeroed) pooled output
                const int pho = a.ho >> 1, pwo = a.wo >> 1;
                if (live && acc > 0.0f && (oh >> 1) < pho && (ow >> 1) < pwo)
                    atomicMax(reinterpret_cast<unsigned*>(a.out) + ((size_t)img * a.c_out + co) * ((size_t)pho * pwo) +
                                  (size_t)(oh >> 1) * pwo + (ow >> 1),
                              __float_as_uint(acc));
                continue;
            }
        }
        if (a.relu) acc = fmaxf(acc, 0.0f);
        if (live) fkw_st(a.out + ((size_t)img * a.c_out + co) * a.ho * a.wo + pix, acc);
    }
}

template <class T>
static hipError_t launch_fkw_t(const DevFkw& f, const T* weight, const ConvShape& s, const T* in, const float* bias,
                               T* out, hipStream_t stream)
{
    FkwArgs<T> a{f.offset, f.reorder, f.index, f.stride, weight, f.masks, in, bias, out,
                 f.num_patterns, s.n, s.c_in, s.c_out, s.h, s.w, s.ho, s.wo, s.stride, s.pad, s.relu, s.pool};
    const unsigned px_blocks = (unsigned)(((long long)s.ho * s.wo + 255) / 256);
    unsigned filters_left = (unsigned)s.c_out;
    // gridDim.y is limited to 65535: walk the filters in slabs
    int32_t s0 = 0;
    while (filters_left) {
        const unsigned fy = filters_left > 65535u ? 65535u : filters_left;
        FkwArgs<T> b = a;
        b.offset += s0;
        b.reorder += s0;
        b.stride += (size_t)s0 * (f.num_patterns + 1);
        dim3 grid(px_blocks, fy, (unsigned)(s.n > 65535 ? 65535 : s.n));
        if (f.taps == 9)
            hipLaunchKernelGGL((fkw_conv_kernel<9, T>), grid, dim3(256), 0, stream, b);
        else
            hipLaunchKernelGGL((fkw_conv_kernel<4, T>), grid, dim3(256), 0, stream, b);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        filters_left -= fy;
        s0 += (int32_t)fy;
    }
    return hipSuccess;
}

hipError_t launch_fkw(const DevFkw& f, const ConvShape& s, const float* in, const float* bias,
                      float* out, hipStream_t stream)
{
    return launch_fkw_t<float>(f, f.weight, s, in, bias, out, stream);
}

hipError_t launch_fkw_f16(const DevFkw& f, const ConvShape& s, const void* in, const float* bias,
                          void* out, hipStream_t stream)
{
    if (s.pool) return hipErrorInvalidValue;
    return launch_fkw_t<__half>(f, static_cast<const __half*>(f.weight_f16), s, static_cast<const __half*>(in), bias,
                                static_cast<__half*>(out), stream);
}

}  // namespace patdnn
