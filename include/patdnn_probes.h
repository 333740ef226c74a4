/*
 * patdnn_probes.h - C ABI of the measurement probes that bench.py times beside the
 * convolution kernels (libpatdnn_probes.so).  They compute nothing of the method.
 * Return 0 on success, 1 for an invalid argument, 4 if the launch failed.
 */
#ifndef PATDNN_PROBES_H
#define PATDNN_PROBES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Copies `bytes` (a multiple of 16; both pointers DEVICE, 16-byte aligned, not
 * overlapping) with a plain kernel, asynchronously on `stream`: it reads and writes
 * exactly `bytes`.  Timed, it gives the achievable HBM stream rate; under
 * rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate those counters.
 */
int32_t patdnn_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * `blocks` workgroups of 256 lanes each run `iters` rounds of 24 independent fp32 FMA
 * chains in registers (plain, non-packed vector FMAs), asynchronously on `stream`.
 * `out` is a DEVICE float the kernel never writes in practice; `*flops` (HOST, may be
 * NULL) receives the floating-point operations the launch performs.
 */
int32_t patdnn_probe_fma(float* out, int32_t blocks, int32_t iters, void* stream, double* flops);

#ifdef __cplusplus
}
#endif
#endif /* PATDNN_PROBES_H */
