// Depthwise pattern-pruned 3x3 convolution (the MobileNet-V2 layers the paper evaluates,
// section 6.1): one four-tap kernel per channel, so the layer does about one flop per byte
// and is bound by HBM bandwidth, not by arithmetic.
//
// Design for that bound: one pass over the input and one over the output.  A lane owns
// four consecutive output pixels of one row (one 16-byte store); per input row that its
// channel's pattern touches it loads 16-byte vectors plus the one or two halo elements
// (predicated, zero outside the image).  Rows are re-read by the lanes of the rows above
// and below, which sit next to each other in the grid and hit the same cache lines, so the
// traffic that reaches HBM is the tensor once.  Channels are walked in the stored filter
// order of the FKW arrays; for one-kernel filters the filter reorder of section 5.2 sorts
// them by pattern, so the lanes of a wavefront share one pattern and skip the same rows
// and taps together (the `if`s on the pattern mask below are then uniform branches).
// Bias and ReLU are fused; the result goes to the original channel `reorder[f]`.
// The same kernel runs on fp32 tensors and on half-precision storage (binary16 weights, input
// and output, fp32 arithmetic in between - the paper's GPU runs keep weights and intermediate
// results in 16 bits, section 6.1): there the bytes, and with them the time, halve.
#include <hip/hip_fp16.h>

#include "kernels.hpp"

namespace patdnn {

template <class T>
struct DwArgs {
    const int32_t* reorder;      // [c] stored filter -> channel
    const int32_t* dw_mask;      // [c] pattern mask of the stored filter's kernel (0: removed)
    const T* dw_weight;          // [c][4] its weights, ascending position
    const T* in;
    const float* bias;
    T* out;
    int32_t c, h, w, ho, wo, wq, pad, relu;
    long long total;             // n * c * ho * wq lanes
    FastDiv div_wq, div_ho, div_c;   // for lane numbers below 2^31 (every realistic launch)
};

// element access: one value, or four consecutive ones with one 16-byte (fp32) / 8-byte
// (binary16) access at an address aligned to that size
__device__ __forceinline__ float ld1(const float* p) { return *p; }
__device__ __forceinline__ float ld1(const __half* p) { return __half2float(*p); }
__device__ __forceinline__ void ld4(const float* p, float& a, float& b, float& c, float& d)
{
    const float4 m = *reinterpret_cast<const float4*>(p);
    a = m.x; b = m.y; c = m.z; d = m.w;
}
__device__ __forceinline__ void ld4(const __half* p, float& a, float& b, float& c, float& d)
{
    const uint2 m = *reinterpret_cast<const uint2*>(p);
    const __half2 lo = *reinterpret_cast<const __half2*>(&m.x), hi = *reinterpret_cast<const __half2*>(&m.y);
    a = __low2float(lo); b = __high2float(lo); c = __low2float(hi); d = __high2float(hi);
}
__device__ __forceinline__ void st1(float* p, float v) { *p = v; }
__device__ __forceinline__ void st1(__half* p, float v) { *p = __float2half_rn(v); }
// NP consecutive elements at an address aligned to NP elements: 16-byte accesses for four
// floats or eight binary16 values
template <int NP>
__device__ __forceinline__ void ldv(const float* p, float* v)
{
#pragma unroll
    for (int k = 0; k < NP; k += 4) ld4(p + k, v[k], v[k + 1], v[k + 2], v[k + 3]);
}
template <int NP>
__device__ __forceinline__ void ldv(const __half* p, float* v)
{
    if constexpr (NP == 8) {
        const uint4 m = *reinterpret_cast<const uint4*>(p);
        const unsigned w[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const __half2 h = *reinterpret_cast<const __half2*>(&w[k]);
            v[2 * k] = __low2float(h);
            v[2 * k + 1] = __high2float(h);
        }
    } else {
        ld4(p, v[0], v[1], v[2], v[3]);
    }
}
template <int NP>
__device__ __forceinline__ void stv(float* p, const float (&v)[NP])
{
#pragma unroll
    for (int k = 0; k < NP; k += 4) *reinterpret_cast<float4*>(p + k) = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
}
template <int NP>
__device__ __forceinline__ void stv(__half* p, const float (&v)[NP])
{
    unsigned w[NP / 2];
#pragma unroll
    for (int k = 0; k < NP / 2; ++k) {
        const __half2 h = __floats2half2_rn(v[2 * k], v[2 * k + 1]);
        w[k] = *reinterpret_cast<const unsigned*>(&h);
    }
    if constexpr (NP == 8) *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    else *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]);
}

// S: stride.  NP: outputs per lane (4, or 8 where the rows allow and the launcher finds it faster).  VEC: rows start aligned to NP elements (w % NP == 0,
// aligned base) -> vector loads.  VST: output rows aligned to NP elements -> one vector store.
template <int S, int NP, bool VEC, bool VST, class T>
__global__ __launch_bounds__(256) void dw_conv_kernel(DwArgs<T> a)
{
    constexpr int NC = (NP - 1) * S + 3;           // input columns under NP outputs
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.total) return;
    // lane number -> (image n, stored channel f, output row oy, group of NP columns xq).  A
    // thread has a dozen FMAs to do, so three 64-bit divisions would be most of its
    // instructions and the kernel would be bound by them instead of by HBM: below 2^31 lanes
    // they are multiplications by launch-time constants.
    int xq, oy, f;
    long long n;
    if (a.total <= 0x7FFFFFFFll) {
        const uint32_t t32 = (uint32_t)t;
        const uint32_t r1 = fast_div(t32, a.div_wq);
        xq = (int)(t32 - r1 * (uint32_t)a.wq);
        const uint32_t r2 = fast_div(r1, a.div_ho);
        oy = (int)(r1 - r2 * (uint32_t)a.ho);
        const uint32_t r3 = fast_div(r2, a.div_c);
        f = (int)(r2 - r3 * (uint32_t)a.c);
        n = r3;
    } else {
        xq = (int)(t % a.wq);
        long long r = t / a.wq;
        oy = (int)(r % a.ho);
        r /= a.ho;
        f = (int)(r % a.c);
        n = r / a.c;
    }
    const int co = a.reorder[f];
    const unsigned mask = (unsigned)a.dw_mask[f];
    float4 wv;
    ld4(a.dw_weight + (size_t)f * 4, wv.x, wv.y, wv.z, wv.w);
    const T* plane = a.in + ((size_t)n * a.c + co) * ((size_t)a.h * a.w);
    const int ox0 = xq * NP;
    const int ix0 = ox0 * S - a.pad;               // input column under (output ox0, tap 0)

    float acc[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const unsigned rowbits = (mask >> (3 * dy)) & 7u;
        if (rowbits == 0) continue;
        const int iy = oy * S + dy - a.pad;
        if (iy < 0 || iy >= a.h) continue;         // zero padding: the row contributes nothing
        const T* row = plane + (size_t)iy * a.w;
        float v[NC];
        if constexpr (VEC) {
            // pad is 0 or 1: columns ix0 + pad .. start a vector
            if (a.pad == 1) {
                v[0] = ((rowbits & 1u) && ix0 >= 0) ? ld1(row + ix0) : 0.0f;
#pragma unroll
                for (int q = 0; q < (NC - 1) / NP; ++q) {
                    const int ix = ix0 + 1 + NP * q;
                    float m[NP];
#pragma unroll
                    for (int k = 0; k < NP; ++k) m[k] = 0.0f;
                    if (ix < a.w) ldv<NP>(row + ix, m);
#pragma unroll
                    for (int k = 0; k < NP; ++k) v[1 + NP * q + k] = m[k];
                }
                if constexpr (S == 1) {
                    const int ix = ix0 + NP + 1;
                    v[NP + 1] = ((rowbits & 4u) && ix < a.w) ? ld1(row + ix) : 0.0f;
                }
            } else {
#pragma unroll
                for (int q = 0; q < (NC + NP - 1) / NP; ++q) {
                    const int ix = ix0 + NP * q;
                    float m[NP];
#pragma unroll
                    for (int k = 0; k < NP; ++k) m[k] = 0.0f;
                    if (ix < a.w) ldv<NP>(row + ix, m);
#pragma unroll
                    for (int k = 0; k < NP; ++k)
                        if (NP * q + k < NC) v[NP * q + k] = m[k];
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                const int ix = ix0 + j;
                v[j] = (ix >= 0 && ix < a.w) ? ld1(row + ix) : 0.0f;
            }
        }
#pragma unroll
        for (int dx = 0; dx < 3; ++dx) {
            if (!((rowbits >> dx) & 1u)) continue;
            // rank of this position among the kept ones = index of its stored weight
            const int rank = __builtin_popcount(mask & ((1u << (3 * dy + dx)) - 1u));
            const float wt = rank == 0 ? wv.x : rank == 1 ? wv.y : rank == 2 ? wv.z : wv.w;
#pragma unroll
            for (int i = 0; i < NP; ++i) acc[i] = fmaf(wt, v[i * S + dx], acc[i]);
        }
    }
    const float b = a.bias ? a.bias[co] : 0.0f;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        acc[i] += b;
        if (a.relu) acc[i] = fmaxf(acc[i], 0.0f);
    }
    T* dst = a.out + (((size_t)n * a.c + co) * a.ho + oy) * (size_t)a.wo + ox0;
    if constexpr (VST) {
        stv<NP>(dst, acc);
    } else {
#pragma unroll
        for (int i = 0; i < NP; ++i)
            if (ox0 + i < a.wo) st1(dst + i, acc[i]);
    }
}

template <class T>
static hipError_t launch_dw_t(const DevFkw& f, const T* weights, const ConvShape& s, const T* in, const float* bias,
                              T* out, hipStream_t stream)
{
    DwArgs<T> a{};
    a.reorder = f.reorder; a.dw_mask = f.dw_mask; a.dw_weight = weights;
    a.in = in; a.bias = bias; a.out = out;
    a.c = s.c_out; a.h = s.h; a.w = s.w; a.ho = s.ho; a.wo = s.wo;
    // eight outputs per lane where every row, in and out, is whole vectors of eight elements
    // (more bytes in flight per lane and half the index arithmetic: 3.0 -> 3.5 TB/s from HBM on
    // the 112x112 fp32 layer); not for fp32 at stride 2, where the seventeen columns under
    // eight outputs made the lanes slower; four otherwise
    constexpr uintptr_t kAlign8 = 8 * sizeof(T) - 1;
    const bool wide = (sizeof(T) == 2 || s.stride == 1) && s.w % 8 == 0 && s.wo % 8 == 0 &&
                      ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & kAlign8) == 0;
    const int np = wide ? 8 : 4;
    a.wq = (s.wo + np - 1) / np; a.pad = s.pad; a.relu = s.relu;
    a.total = (long long)s.n * s.c_out * s.ho * a.wq;
    a.div_wq = make_fast_div((uint32_t)a.wq);
    a.div_ho = make_fast_div((uint32_t)a.ho);
    a.div_c = make_fast_div((uint32_t)a.c);
    const long long blocks = (a.total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    // vector loads need every row to start aligned to four elements and to be read in whole
    // vectors: the columns a lane reads beyond its last tap stay inside the row when w % 4 == 0
    constexpr uintptr_t kAlign = 4 * sizeof(T) - 1;
    const bool vec = s.w % 4 == 0 && (reinterpret_cast<uintptr_t>(in) & kAlign) == 0;
    const bool vst = s.wo % 4 == 0 && (reinterpret_cast<uintptr_t>(out) & kAlign) == 0;
    const dim3 grid((unsigned)blocks), block(256);
#define PATDNN_DW_LAUNCH(S, V, W) hipLaunchKernelGGL((dw_conv_kernel<S, 4, V, W, T>), grid, block, 0, stream, a)
    if (wide) {
        if (s.stride == 1) hipLaunchKernelGGL((dw_conv_kernel<1, 8, true, true, T>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((dw_conv_kernel<2, 8, true, true, T>), grid, block, 0, stream, a);
    } else if (s.stride == 1) {
        if (vec && vst) PATDNN_DW_LAUNCH(1, true, true);
        else if (vec) PATDNN_DW_LAUNCH(1, true, false);
        else if (vst) PATDNN_DW_LAUNCH(1, false, true);
        else PATDNN_DW_LAUNCH(1, false, false);
    } else {
        if (vec && vst) PATDNN_DW_LAUNCH(2, true, true);
        else if (vec) PATDNN_DW_LAUNCH(2, true, false);
        else if (vst) PATDNN_DW_LAUNCH(2, false, true);
        else PATDNN_DW_LAUNCH(2, false, false);
    }
#undef PATDNN_DW_LAUNCH
    return hipGetLastError();
}

hipError_t launch_dw(const DevFkw& f, const ConvShape& s, const float* in, const float* bias,
                     float* out, hipStream_t stream)
{
    return launch_dw_t<float>(f, f.dw_weight, s, in, bias, out, stream);
}

hipError_t launch_dw_f16(const DevFkw& f, const ConvShape& s, const void* in, const float* bias,
                         void* out, hipStream_t stream)
{
    return launch_dw_t<__half>(f, static_cast<const __half*>(f.dw_weight_f16), s, static_cast<const __half*>(in), bias,
                               static_cast<__half*>(out), stream);
}

}  // namespace patdnn
