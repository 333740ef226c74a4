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
#include "kernels.hpp"

namespace patdnn {

struct DwArgs {
    const int32_t* reorder;      // [c] stored filter -> channel
    const int32_t* dw_mask;      // [c] pattern mask of the stored filter's kernel (0: removed)
    const float* dw_weight;      // [c][4] its weights, ascending position
    const float* in;
    const float* bias;
    float* out;
    int32_t c, h, w, ho, wo, wq, pad, relu;
    long long total;             // n * c * ho * wq lanes
};

// S: stride.  VEC: rows start 16-byte aligned (w % 4 == 0, aligned base) -> vector loads.
// VST: output rows 16-byte aligned (wo % 4 == 0, aligned base) -> one vector store.
template <int S, bool VEC, bool VST>
__global__ __launch_bounds__(256) void dw_conv_kernel(DwArgs a)
{
    constexpr int NC = 3 * S + 3;                  // input columns under four outputs: 6 or 9
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.total) return;
    const int xq = (int)(t % a.wq);
    long long r = t / a.wq;
    const int oy = (int)(r % a.ho);
    r /= a.ho;
    const int f = (int)(r % a.c);
    const long long n = r / a.c;
    const int co = a.reorder[f];
    const unsigned mask = (unsigned)a.dw_mask[f];
    const float4 wv = reinterpret_cast<const float4*>(a.dw_weight)[f];
    const float* plane = a.in + ((size_t)n * a.c + co) * ((size_t)a.h * a.w);
    const int ox0 = xq * 4;
    const int ix0 = ox0 * S - a.pad;               // input column under (output ox0, tap 0)

    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const unsigned rowbits = (mask >> (3 * dy)) & 7u;
        if (rowbits == 0) continue;
        const int iy = oy * S + dy - a.pad;
        if (iy < 0 || iy >= a.h) continue;         // zero padding: the row contributes nothing
        const float* row = plane + (size_t)iy * a.w;
        float v[NC];
        if constexpr (VEC) {
            // pad is 0 or 1: columns ix0 + pad .. are 16-byte aligned
            if (a.pad == 1) {
                v[0] = ((rowbits & 1u) && ix0 >= 0) ? row[ix0] : 0.0f;
#pragma unroll
                for (int q = 0; q < (NC - 1) / 4; ++q) {
                    const int ix = ix0 + 1 + 4 * q;
                    float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (ix < a.w) m = *reinterpret_cast<const float4*>(row + ix);
                    v[1 + 4 * q] = m.x; v[2 + 4 * q] = m.y; v[3 + 4 * q] = m.z; v[4 + 4 * q] = m.w;
                }
                if constexpr (S == 1) {
                    const int ix = ix0 + 5;
                    v[5] = ((rowbits & 4u) && ix < a.w) ? row[ix] : 0.0f;
                }
            } else {
#pragma unroll
                for (int q = 0; q < (NC + 3) / 4; ++q) {
                    const int ix = ix0 + 4 * q;
                    float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (ix < a.w) m = *reinterpret_cast<const float4*>(row + ix);
                    if (4 * q + 0 < NC) v[4 * q + 0] = m.x;
                    if (4 * q + 1 < NC) v[4 * q + 1] = m.y;
                    if (4 * q + 2 < NC) v[4 * q + 2] = m.z;
                    if (4 * q + 3 < NC) v[4 * q + 3] = m.w;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                const int ix = ix0 + j;
                v[j] = (ix >= 0 && ix < a.w) ? row[ix] : 0.0f;
            }
        }
#pragma unroll
        for (int dx = 0; dx < 3; ++dx) {
            if (!((rowbits >> dx) & 1u)) continue;
            // rank of this position among the kept ones = index of its stored weight
            const int rank = __builtin_popcount(mask & ((1u << (3 * dy + dx)) - 1u));
            const float wt = rank == 0 ? wv.x : rank == 1 ? wv.y : rank == 2 ? wv.z : wv.w;
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = fmaf(wt, v[i * S + dx], acc[i]);
        }
    }
    const float b = a.bias ? a.bias[co] : 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc[i] += b;
        if (a.relu) acc[i] = fmaxf(acc[i], 0.0f);
    }
    float* dst = a.out + (((size_t)n * a.c + co) * a.ho + oy) * (size_t)a.wo + ox0;
    if constexpr (VST) {
        *reinterpret_cast<float4*>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (ox0 + i < a.wo) dst[i] = acc[i];
    }
}

hipError_t launch_dw(const DevFkw& f, const ConvShape& s, const float* in, const float* bias,
                     float* out, hipStream_t stream)
{
    DwArgs a{};
    a.reorder = f.reorder; a.dw_mask = f.dw_mask; a.dw_weight = f.dw_weight;
    a.in = in; a.bias = bias; a.out = out;
    a.c = s.c_out; a.h = s.h; a.w = s.w; a.ho = s.ho; a.wo = s.wo;
    a.wq = (s.wo + 3) / 4; a.pad = s.pad; a.relu = s.relu;
    a.total = (long long)s.n * s.c_out * s.ho * a.wq;
    const long long blocks = (a.total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return hipErrorInvalidValue;
    // vector loads need every row to start 16-byte aligned and to be read in whole vectors:
    // the columns a lane reads beyond its last tap stay inside the row when w % 4 == 0
    const bool vec = s.w % 4 == 0 && (reinterpret_cast<uintptr_t>(in) & 15u) == 0;
    const bool vst = s.wo % 4 == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
    const dim3 grid((unsigned)blocks), block(256);
#define PATDNN_DW_LAUNCH(S, V, T) hipLaunchKernelGGL((dw_conv_kernel<S, V, T>), grid, block, 0, stream, a)
    if (s.stride == 1) {
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

}  // namespace patdnn
