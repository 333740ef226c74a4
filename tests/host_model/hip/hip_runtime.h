// Stand-in for <hip/hip_runtime.h> - TEST INFRASTRUCTURE.
//
// With this header first on the include path, csrc/kernel_tiled.hip compiles as plain
// C++ for the host: one OS thread per GPU thread of a workgroup (pthread barrier for
// __syncthreads), workgroups one after another, LDS as a poisoned array, buffer loads
// with the range check of a raw buffer descriptor.  Every access the kernel makes to
// LDS and to its tensors is bounds-checked here, so that a new tile geometry is run on
// the CPU before it ever reaches a GPU.  The inline-assembly interpreter is replaced by
// a C++ walk of the same step stream (hostmodel_walk).
#pragma once

#include <pthread.h>

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __shared__
#define address_space(x)

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
typedef int hipError_t;
typedef void* hipStream_t;
constexpr hipError_t hipSuccess = 0, hipErrorInvalidValue = 1;
constexpr int hipFuncAttributeMaxDynamicSharedMemorySize = 8;
struct alignas(16) float4 { float x, y, z, w; };
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
// a small machine, so that the launches of the tests span several rounds of workgroups
enum hipDeviceAttribute_t { hipDeviceAttributeMultiprocessorCount = 0 };
inline hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 2; return hipSuccess; }
inline hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int* n, const void*, int, size_t) { *n = 3; return hipSuccess; }

namespace hostmodel {

constexpr size_t kLdsFloats = 160 * 1024 / 4;

struct State {
    size_t lds_floats = 0;             // dynamic LDS of the current launch
    const float* in = nullptr;         // input tensor and its size, for range checks
    size_t in_floats = 0;
    float* out = nullptr;
    size_t out_floats = 0;
    long errors = 0;
    std::string first_error;
    pthread_barrier_t barrier;
    pthread_barrier_t wave_barrier[16];   // one per wavefront of the workgroup (lane exchanges)
    int exchange[16][64];
    pthread_mutex_t lock = PTHREAD_MUTEX_INITIALIZER;
};
State& state();
void fail(const char* what, long a = 0, long b = 0);

}  // namespace hostmodel

extern thread_local dim3 threadIdx;
extern dim3 blockIdx, blockDim, gridDim;

namespace patdnn { extern float lds[]; }

inline void __syncthreads() { pthread_barrier_wait(&hostmodel::state().barrier); }
inline int min(int a, int b) { return a < b ? a : b; }
inline int max(int a, int b) { return a > b ? a : b; }

// hardware fp32 atomic add: workgroups run one after another here and the lanes of a
// workgroup add to distinct elements, so a locked add is enough
inline float unsafeAtomicAdd(float* p, float v)
{
    hostmodel::State& st = hostmodel::state();
    if (p < st.out || p >= st.out + st.out_floats) {
        hostmodel::fail("atomic add outside the output tensor", p - st.out);
        return 0.0f;
    }
    pthread_mutex_lock(&st.lock);
    const float old = *p;
    *p = old + v;
    pthread_mutex_unlock(&st.lock);
    return old;
}

// unsigned atomic max on the output tensor (the fused pooling epilogue folds float bits in)
inline unsigned atomicMax(unsigned* p, unsigned v)
{
    hostmodel::State& st = hostmodel::state();
    float* fp = reinterpret_cast<float*>(p);
    if (fp < st.out || fp >= st.out + st.out_floats) {
        hostmodel::fail("atomic max outside the output tensor", fp - st.out);
        return 0u;
    }
    pthread_mutex_lock(&st.lock);
    const unsigned old = *p;
    if (v > old) *p = v;
    pthread_mutex_unlock(&st.lock);
    return old;
}
inline unsigned __float_as_uint(float f)
{
    unsigned u;
    __builtin_memcpy(&u, &f, 4);
    return u;
}

inline int __float_as_int(float f)
{
    int i;
    __builtin_memcpy(&i, &f, 4);
    return i;
}
inline float __int_as_float(int i)
{
    float f;
    __builtin_memcpy(&f, &i, 4);
    return f;
}

// ds_bpermute_b32: every lane of the wavefront takes `value` of lane (addr / 4) % 64.  All 64
// lanes (OS threads) of the wavefront must call it together, as on the hardware with a full
// EXEC mask; a lane that stayed away would leave the others at the barrier, so a kernel
// that calls it under a per-lane condition hangs here instead of passing by luck.
inline int __builtin_amdgcn_ds_bpermute(int addr, int value)
{
    hostmodel::State& st = hostmodel::state();
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    st.exchange[wave][lane] = value;
    pthread_barrier_wait(&st.wave_barrier[wave]);
    const int got = st.exchange[wave][((unsigned)addr >> 2) & 63];
    pthread_barrier_wait(&st.wave_barrier[wave]);
    return got;
}

#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_s_waitcnt(x) ((void)0)
#define __builtin_amdgcn_s_setprio(x) ((void)0)     // issue arbitration only: no effect on results

// ---- raw buffer descriptor and the LDS-direct load
struct __amdgpu_buffer_rsrc_t {
    const char* base;
    unsigned num_records;
};
#define __builtin_amdgcn_make_buffer_rsrc(ptr, stride, num, flags) \
    __amdgpu_buffer_rsrc_t { (const char*)(ptr), (unsigned)(num) }

// The wavefront writes 64 consecutive dwords at `lds_dst`; this thread is lane tid & 63.
inline void __builtin_amdgcn_raw_ptr_buffer_load_lds(__amdgpu_buffer_rsrc_t r, float* lds_dst, int size,
                                                    int voffset, int soffset, int offset, int aux)
{
    using namespace hostmodel;
    State& st = state();
    (void)aux;
    if (size != 4 || soffset != 0 || offset != 0) fail("buffer load form not modelled");
    float* dst = lds_dst + (threadIdx.x & 63);
    const ptrdiff_t at = dst - patdnn::lds;
    if (at < 0 || (size_t)at >= st.lds_floats) {
        fail("LDS-direct load writes outside the launch's LDS", at, (long)st.lds_floats);
        return;
    }
    const unsigned vo = (unsigned)voffset;
    float v = 0.0f;                                          // out of range reads as zero
    if ((unsigned long long)vo + 4 <= r.num_records) {
        const char* p = r.base + vo;
        const char* lo = (const char*)st.in;
        if (p < lo || p + 4 > lo + 4 * st.in_floats || (p - lo) % 4) {
            fail("buffer load inside the descriptor's range but outside the input tensor", p - lo);
            return;
        }
        std::memcpy(&v, p, 4);
    }
    *dst = v;
}

// ---- launch: workgroups one after another, one OS thread per GPU thread
template <class... Args>
void hostmodel_launch(void (*kernel)(Args...), dim3 grid, dim3 block, size_t lds_bytes, Args... args)
{
    using namespace hostmodel;
    State& st = state();
    if (lds_bytes > 4 * kLdsFloats) { fail("more dynamic LDS than a CU has", (long)lds_bytes); return; }
    st.lds_floats = lds_bytes / 4;
    gridDim = grid;
    blockDim = block;
    for (unsigned by = 0; by < grid.y; ++by)
    for (unsigned b = 0; b < grid.x; ++b) {
        blockIdx = dim3(b, by);
        const uint32_t poison = 0x7FC0DEADu;                 // NaN: reading unstaged LDS shows in the output
        for (size_t i = 0; i < kLdsFloats; ++i) std::memcpy(&patdnn::lds[i], &poison, 4);
        pthread_barrier_init(&st.barrier, nullptr, block.x);
        for (unsigned w = 0; w < block.x / 64; ++w) pthread_barrier_init(&st.wave_barrier[w], nullptr, 64);
        std::vector<std::thread> threads;
        for (unsigned t = 0; t < block.x; ++t)
            threads.emplace_back([=]() {
                threadIdx = dim3(t);
                kernel(args...);
            });
        for (auto& th : threads) th.join();
        pthread_barrier_destroy(&st.barrier);
        for (unsigned w = 0; w < block.x / 64; ++w) pthread_barrier_destroy(&st.wave_barrier[w]);
    }
}
#define hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, ...) \
    hostmodel_launch(kernel, grid, block, lds_bytes, __VA_ARGS__)

// ---- the step interpreter, walked in C++ (one lane)
struct HostmodelGeo {
    int G, PR, PC, S, WR, WC, rowp;          // rowp: floats between window rows in LDS
    unsigned block_bytes, table_off, ctrl_bytes, records;
    int sets, threaded;
};
void hostmodel_walk(const HostmodelGeo& g, float* acc, unsigned lane_lds, const uint32_t* stream,
                    unsigned entry);
