// Device-side views of an encoded layer and the launchers of each kernel family.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "layout.hpp"

namespace patdnn {

struct ConvShape {
    int32_t n, c_in, c_out, h, w, ho, wo, stride, pad, relu;
    // pool != 0: ReLU, then 2x2 max pooling with stride 2 (floor), fused into the epilogue.
    // The output tensor is [n][c_out][ho/2][wo/2] and must hold zeros when the kernel
    // starts: every lane folds its values in with an unsigned integer atomic max on the
    // float bits, which orders non-negative floats like the floats themselves.
    int32_t pool = 0;
    // Zero-fill hand-off between consecutive launches of a stack (all optional).  The launches
    // that add into their target with atomics (split, pooled) need it zeroed beforehand, which
    // costs a kernel launch of its own; a launch that ends with a finishing kernel can clear
    // the next launch's target in that same kernel instead.
    //   pre_zeroed / pre_zeroed_count: a region that already holds zeros on entry; a zero fill of
    //     exactly that region (same start, no more floats) is skipped.
    //   zero_next / zero_next_count: a region to clear in this launch's finishing kernel, if it
    //     has one and the region is not one the kernel still reads; *zero_next_done is set when
    //     it was cleared (left alone otherwise).
    const float* pre_zeroed = nullptr;
    size_t pre_zeroed_count = 0;
    float* zero_next = nullptr;
    size_t zero_next_count = 0;
    bool* zero_next_done = nullptr;
};

// Fills `count` floats with zero (a kernel, so that it can be captured into a HIP graph).
hipError_t launch_fill_zero(float* p, size_t count, hipStream_t stream);

// Floats between the partial-sum buffers of a split launch whose output has `total` floats (a
// launch with `ksplit` slices stores to buffers if its scratch holds ksplit of them).
size_t split_slice_stride(size_t total);

// Division of a value below 2^31 by a launch-time constant d >= 1 without the divider loop:
// with l = ceil(log2 d) and m = ceil(2^(31+l) / d) (which fits 32 bits), floor(n / d) =
// (n * m) >> (31 + l) exactly for every n < 2^31 (the error term n * (m*d - 2^(31+l)) /
// (d * 2^(31+l)) stays below 2^-l <= 1/d).  The tiled kernel divides band numbers by the bands per
// image row and column seven times per thread before it can start; the depthwise kernel, which
// has a dozen FMAs per thread, spends most of its instructions on turning a thread number into
// (image, channel, row, column).
struct FastDiv {
    uint32_t m, shift;
};
inline FastDiv make_fast_div(uint32_t d)
{
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    const uint64_t p = 1ull << (31 + l);
    return FastDiv{(uint32_t)((p + d - 1) / d), 31 + l};
}
__host__ __device__ __forceinline__ uint32_t fast_div(uint32_t n, FastDiv f)
{
    return (uint32_t)(((uint64_t)n * f.m) >> f.shift);
}


// FKW arrays on the device (paper section 5.3).
struct DevFkw {
    const int32_t* offset = nullptr;
    const int32_t* reorder = nullptr;
    const int32_t* index = nullptr;
    const int32_t* stride = nullptr;
    const float* weight = nullptr;
    const uint16_t* masks = nullptr;
    int32_t num_patterns = 0;
    int32_t taps = 4;
    // depthwise layers: per stored filter, the pattern mask of its one kernel (0 if the
    // kernel was removed) and its four weights
    const int32_t* dw_mask = nullptr;
    const float* dw_weight = nullptr;
    // the weights once more as IEEE binary16 (round to nearest even), for the
    // half-precision-storage entry point: `weight` and `dw_weight` element for element
    const void* weight_f16 = nullptr;
    const void* dw_weight_f16 = nullptr;
};

// Filter-group layout on the device: record streams (sparse) or 9-tap weights (dense).
struct DevTiled {
    int32_t G = 0;
    int32_t num_groups = 0;
    int32_t ck = 0;            // input channels staged per LDS pass (fixes the chunking of the streams)
    int32_t num_chunks = 0;
    const int32_t* slot_channel = nullptr;
    const uint32_t* chunk_ptr = nullptr;   // [num_groups][num_chunks] first step of a chunk | entry block << 28
    const uint32_t* steps = nullptr;       // [steps][kStepDwords]
    const float* w9 = nullptr;
};

// Filter-major walk of the FKW arrays, one lane per output pixel.
hipError_t launch_fkw(const DevFkw& f, const ConvShape& s, const float* in, const float* bias,
                      float* out, hipStream_t stream);

// The comparison kernels' views of a layer (kernel_compare.hip): the layer before
// filter-kernel reorder, and as a CSR matrix.
struct DevCompare {
    const int32_t* row_ptr = nullptr;
    const int32_t* col = nullptr;
    const int32_t* kmask = nullptr;
    const float* val = nullptr;
};
hipError_t launch_compare(bool csr, const DevCompare& d, const ConvShape& s, const float* in, const float* bias,
                          float* out, hipStream_t stream);

// Depthwise layers: one pass over input and output, 16-byte accesses, four outputs per lane.
hipError_t launch_dw(const DevFkw& f, const ConvShape& s, const float* in, const float* bias,
                     float* out, hipStream_t stream);
// The same two kernels on binary16 tensors and weights (fp32 arithmetic, fp32 bias).
hipError_t launch_dw_f16(const DevFkw& f, const ConvShape& s, const void* in, const float* bias,
                         void* out, hipStream_t stream);
hipError_t launch_fkw_f16(const DevFkw& f, const ConvShape& s, const void* in, const float* bias,
                          void* out, hipStream_t stream);

// ---------------------------------------------------------------------------
// Tiled kernels: compile-time geometry per variant, run-time launch parameters.
// ---------------------------------------------------------------------------
struct TiledVariant {
    const char* name;
    int32_t G;        // filters per group (one group per wavefront)
    int32_t PR, PC;   // output patch per lane (rows x columns)
    int32_t S;        // stride
    int32_t TGX;      // lanes across a band; a wavefront covers 64/TGX bands
    bool dense;       // nine taps, every kernel present
    bool double_window;   // two sets of window registers: the next channel's window loads early
    bool threaded;        // every code block jumps straight to the next kernel's block
    bool experimental;    // not yet measured on hardware: never chosen by default or by the tuner
    int32_t mode;         // MODE bits: 0-3 the interpreter's (gen_dispatch.py), 4 one staging buffer
    int32_t lds_buffers;  // staging buffers of `ck` channels each (1 or 2)
    int32_t lds_floats_per_channel;   // LDS floats one staged channel takes
    int32_t stage_elems;              // elements staged per channel (without bank padding)
    int32_t max_slots;                // staging elements per thread the kernel can hold
    // code-table geometry of the step interpreter (sparse variants)
    uint32_t block_bytes;             // size of one (set, slot, pattern) block
    uint32_t table_off;               // offset of block 0 from the code base
    uint32_t ctrl_bytes;              // control block k sits at k*ctrl_bytes
    uint32_t records;                 // kernels per step
    // ksplit > 1 (sparse variants): slices of the input channels on gridDim.y.  `scratch` (DEVICE,
    // 16-byte aligned, `scratch_floats` floats, may be NULL): with room for ksplit buffers of
    // split_slice_stride([n][c_out][ho][wo]) floats every slice stores its partial sums to its
    // own buffer and a finishing kernel adds them up; otherwise the slices are summed with
    // atomics, in the output or - with fused pooling, which then needs [n][c_out][ho][wo]
    // floats of scratch - in `scratch`, and a finishing kernel writes the pooled output.
    hipError_t (*launch)(const DevTiled&, const ConvShape&, const float*, const float*, float*,
                         int32_t waves, int32_t ksplit, float* scratch, size_t scratch_floats, hipStream_t);
};

// Device check that s_movrels_b32 / _b64 behave as the threaded interpreter assumes.
bool movrel_selftest(std::string& err);

int num_tiled_variants();
const TiledVariant& tiled_variant(int i);

}  // namespace patdnn
