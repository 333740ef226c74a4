// Comparison kernels of the paper's evaluation, not on the product path: they exist so that
// the per-layer breakdown of section 6.3 (what filter-kernel reorder, load-redundancy
// elimination and tuning each buy) and the CSR control of section 6.2 can be re-measured on
// this GPU.  Both use one lane per output pixel, like the reorder-only FKW kernel, so that the
// only difference between "noopt" and "fkw" is the reorder.
//
//   noopt  the pruned layer before filter-kernel reorder (section 5.2, "No-opt"): filters in
//          their original order, the kernels of a filter in input-channel order, and the pattern
//          of every kernel decided inside the inner loop (a branch per position of the 3x3
//          window per kernel) - the control flow the reorder removes.
//   csr    the layer as a conventional compressed-sparse-row matrix [c_out][c_in*9]
//          (section 5.3): one column index per stored weight, decoded per weight into
//          channel and tap.
#include "kernels.hpp"

namespace patdnn {

struct CompareArgs {
    const int32_t* row_ptr;      // [c_out+1] kernels (noopt) or weights (csr) per filter, cumulative
    const int32_t* col;          // noopt: input channel per kernel; csr: ci*9 + 3*kh + kw per weight
    const int32_t* kmask;        // noopt: pattern mask per kernel
    const float* val;            // noopt: [kernels][4]; csr: [weights]
    const float* in;
    const float* bias;
    float* out;
    int32_t n, c_in, c_out, h, w, ho, wo, conv_stride, pad, relu;
};

__global__ __launch_bounds__(256) void noopt_conv_kernel(CompareArgs a)
{
    const int co = blockIdx.y;
    const int pix = blockIdx.x * 256 + threadIdx.x;
    if (pix >= a.ho * a.wo) return;
    const int oh = pix / a.wo, ow = pix - oh * a.wo;
    const size_t plane = (size_t)a.h * a.w;
    for (int img = blockIdx.z; img < a.n; img += gridDim.z) {
        const float* in_img = a.in + (size_t)img * a.c_in * plane;
        float acc = 0.0f;
        for (int32_t k = a.row_ptr[co]; k < a.row_ptr[co + 1]; ++k) {
            const float* src = in_img + (size_t)a.col[k] * plane;
            const unsigned m = (unsigned)a.kmask[k];
            const float* wk = a.val + (size_t)k * 4;
            int t = 0;
            for (int pos = 0; pos < 9; ++pos) {
                if (!((m >> pos) & 1u)) continue;               // which taps this kernel has: decided here
                const int kh = pos / 3, kw = pos - 3 * kh;
                const int ih = oh * a.conv_stride + kh - a.pad, iw = ow * a.conv_stride + kw - a.pad;
                const float x = (ih >= 0 && ih < a.h && iw >= 0 && iw < a.w) ? src[(size_t)ih * a.w + iw] : 0.0f;
                acc = fmaf(wk[t++], x, acc);
            }
        }
        if (a.bias) acc += a.bias[co];
        if (a.relu) acc = fmaxf(acc, 0.0f);
        a.out[((size_t)img * a.c_out + co) * a.ho * a.wo + pix] = acc;
    }
}

__global__ __launch_bounds__(256) void csr_conv_kernel(CompareArgs a)
{
    const int co = blockIdx.y;
    const int pix = blockIdx.x * 256 + threadIdx.x;
    if (pix >= a.ho * a.wo) return;
    const int oh = pix / a.wo, ow = pix - oh * a.wo;
    const size_t plane = (size_t)a.h * a.w;
    for (int img = blockIdx.z; img < a.n; img += gridDim.z) {
        const float* in_img = a.in + (size_t)img * a.c_in * plane;
        float acc = 0.0f;
        for (int32_t k = a.row_ptr[co]; k < a.row_ptr[co + 1]; ++k) {
            const int c = a.col[k];
            const int ci = c / 9, pos = c - 9 * ci;
            const int kh = pos / 3, kw = pos - 3 * kh;
            const int ih = oh * a.conv_stride + kh - a.pad, iw = ow * a.conv_stride + kw - a.pad;
            const float x = (ih >= 0 && ih < a.h && iw >= 0 && iw < a.w) ? in_img[(size_t)ci * plane + (size_t)ih * a.w + iw] : 0.0f;
            acc = fmaf(a.val[k], x, acc);
        }
        if (a.bias) acc += a.bias[co];
        if (a.relu) acc = fmaxf(acc, 0.0f);
        a.out[((size_t)img * a.c_out + co) * a.ho * a.wo + pix] = acc;
    }
}

hipError_t launch_compare(bool csr, const DevCompare& d, const ConvShape& s, const float* in, const float* bias,
                          float* out, hipStream_t stream)
{
    if (s.c_out > 65535) return hipErrorInvalidValue;
    CompareArgs a{d.row_ptr, d.col, d.kmask, d.val, in, bias, out,
                  s.n, s.c_in, s.c_out, s.h, s.w, s.ho, s.wo, s.stride, s.pad, s.relu};
    const dim3 grid((unsigned)(((long long)s.ho * s.wo + 255) / 256), (unsigned)s.c_out,
                    (unsigned)(s.n > 65535 ? 65535 : s.n));
    if (csr) hipLaunchKernelGGL(csr_conv_kernel, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(noopt_conv_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace patdnn
