// Threaded dispatch reads the next record with scalar relative moves (s_movrels_b32 / _b64,
// index in M0) and then JUMPS to an address taken from what it read.  Before the first
// layout of a threaded variant is built, the instruction's behaviour on this device is
// checked with a kernel that only moves registers and stores the results: if the moves do
// not return what the generated code assumes, the threaded variants are refused instead
// of jumping to a wrong address.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "kernels.hpp"

namespace patdnn {

__global__ __launch_bounds__(64) void movrel_selftest_kernel(uint32_t* out)
{
    uint32_t a, b0, b1, c, m0_after;
    asm volatile(
        "s_mov_b32 s60, m0\n"
        "s_mov_b32 s40, 0x1000\n"
        "s_mov_b32 s41, 0x1001\n"
        "s_mov_b32 s42, 0x1002\n"
        "s_mov_b32 s43, 0x1003\n"
        "s_mov_b32 s44, 0x1004\n"
        "s_mov_b32 s45, 0x1005\n"
        "s_mov_b32 s46, 0x1006\n"
        "s_mov_b32 s47, 0x1007\n"
        "s_mov_b32 s48, 0x1008\n"
        "s_mov_b32 s49, 0x1009\n"
        "s_mov_b32 s50, 0x100a\n"
        "s_mov_b32 s51, 0x100b\n"
        "s_mov_b32 m0, 6\n"
        "s_nop 0\n"
        "s_movrels_b32 %[a], s40\n"              // s46
        "s_movrels_b64 s[62:63], s[40:41]\n"     // s46, s47
        "s_add_u32 m0, m0, 4\n"
        "s_nop 0\n"
        "s_movrels_b32 %[c], s41\n"              // s51
        "s_mov_b32 %[b0], s62\n"
        "s_mov_b32 %[b1], s63\n"
        "s_mov_b32 %[m], m0\n"
        "s_mov_b32 m0, s60\n"
        : [a] "=s"(a), [b0] "=s"(b0), [b1] "=s"(b1), [c] "=s"(c), [m] "=s"(m0_after)
        :
        : "s40", "s41", "s42", "s43", "s44", "s45", "s46", "s47", "s48", "s49", "s50", "s51", "s60", "s62", "s63",
          "scc");
    if (threadIdx.x == 0) {
        out[0] = a;
        out[1] = b0;
        out[2] = b1;
        out[3] = c;
        out[4] = m0_after;
    }
}

// true if scalar relative moves behave as the threaded interpreter assumes; the result of
// the first call on a device is kept for the process.
bool movrel_selftest(std::string& err)
{
    static int cached = -1;            // -1 not run, 0 failed, 1 passed
    static std::string cached_err;
    if (cached < 0) {
        cached = 0;
        uint32_t* dev = nullptr;
        uint32_t host[5] = {0, 0, 0, 0, 0};
        hipError_t e = hipMalloc(&dev, sizeof(host));
        if (e == hipSuccess) e = hipMemset(dev, 0, sizeof(host));
        if (e == hipSuccess) {
            hipLaunchKernelGGL(movrel_selftest_kernel, dim3(1), dim3(64), 0, nullptr, dev);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpy(host, dev, sizeof(host), hipMemcpyDeviceToHost);
        if (dev) (void)hipFree(dev);
        if (e != hipSuccess) {
            cached_err = std::string("scalar relative move self-test could not run: ") + hipGetErrorString(e);
        } else if (host[0] != 0x1006 || host[1] != 0x1006 || host[2] != 0x1007 || host[3] != 0x100b || host[4] != 10) {
            char buf[160];
            snprintf(buf, sizeof(buf), "scalar relative moves returned %x %x %x %x (m0 %u), expected 1006 1006 1007 100b (m0 10)",
                     host[0], host[1], host[2], host[3], host[4]);
            cached_err = buf;
        } else {
            cached = 1;
        }
    }
    err = cached_err;
    return cached == 1;
}

}  // namespace patdnn
