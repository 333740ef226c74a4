/*
 * CPU oracle for pattern- and connectivity-pruned 3x3 convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against; nothing in the product path may call it.
 * It shares no code with the HIP library.
 *
 * What it computes (paper section 2.1 for the CONV layer and the ReLU that
 * follows it; section 3.1 / 4.2 for the two pruning constraints):
 *
 *   Wm[co][ci][kh][kw] = W[co][ci][kh][kw]   if kernel (co,ci) survives connectivity
 *                                            pruning AND position 3*kh+kw belongs to
 *                                            the kernel's pattern
 *                      = 0                   otherwise
 *   out[n][co][oh][ow] = act( bias[co] + sum_ci sum_kh sum_kw
 *                             Wm[co][ci][kh][kw] * in[n][ci][oh*s+kh-p][ow*s+kw-p] )
 *
 * with in[] = 0 outside the image, act = max(.,0) when ReLU is fused, and
 * H_out = floor((H + 2p - 3)/s) + 1.  The operation is cross-correlation (no
 * kernel flip), the convention of the framework the paper trains in
 * (section 4.3).  A depthwise layer has one kernel per filter and ci == co.
 * A "dense" layer keeps all nine taps of every kernel (the paper leaves the
 * first layer unpruned, section 4.2).
 *
 * All arithmetic is IEEE double; fp32 inputs are widened exactly.  The sum runs
 * in the fixed order (ci, kh, kw).  Threads (OpenMP) split (n, co) only, so
 * every output value is computed by one thread in that order.
 *
 * The reorder / compact-storage / redundancy-elimination machinery of section 5
 * changes only the order of operations, so it is deliberately absent here.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t c_out, c_in;       /* depthwise: c_in == c_out, one kernel per filter */
    int32_t depthwise;         /* 0 / 1 */
    int32_t dense;             /* 1: ignore ids, keep all 9 taps of surviving kernels */
    int32_t stride, pad;
    int32_t num_patterns;
    int32_t relu;
    int32_t skip_removed;      /* 1: do not visit kernels removed by connectivity pruning
                                  (adds no +0.0 products; same value up to the sign of zero) */
    int32_t nthreads;          /* <= 0: OpenMP default */
} patdnn_ref_desc;

static int out_dim(int in, int pad, int stride) { return (in + 2 * pad - 3) / stride + 1; }

/* value of one output element; the definition above, nothing else */
static double one_output(const patdnn_ref_desc* d, const float* w, const uint8_t* ids,
                         const uint8_t* kmask, const uint16_t* pmasks, const float* in,
                         int h, int wd, const float* bias, int n, int co, int oh, int ow)
{
    const int kpf = d->depthwise ? 1 : d->c_in;   /* kernels per filter */
    double acc = bias ? (double)bias[co] : 0.0;
    for (int k = 0; k < kpf; ++k) {
        const int ci = d->depthwise ? co : k;
        const size_t kidx = (size_t)co * kpf + k;
        const int kept = kmask ? (kmask[kidx] != 0) : 1;
        if (!kept && d->skip_removed) continue;
        const unsigned pm = !kept ? 0u : (d->dense ? 0x1FFu : pmasks[ids[kidx]]);
        const float* wk = w + kidx * 9;
        const float* plane = in + ((size_t)n * d->c_in + ci) * (size_t)h * wd;
        for (int kh = 0; kh < 3; ++kh) {
            for (int kw = 0; kw < 3; ++kw) {
                const int in_pattern = (pm >> (3 * kh + kw)) & 1u;
                const double wm = (kept && in_pattern) ? (double)wk[3 * kh + kw] : 0.0;
                const int ih = oh * d->stride + kh - d->pad;
                const int iw = ow * d->stride + kw - d->pad;
                const double x = (ih >= 0 && ih < h && iw >= 0 && iw < wd)
                                     ? (double)plane[(size_t)ih * wd + iw] : 0.0;
                acc += wm * x;
            }
        }
    }
    if (d->relu && acc < 0.0) acc = 0.0;
    return acc;
}

static int check(const patdnn_ref_desc* d, const float* w, const uint8_t* ids,
                 const uint8_t* kmask, const uint16_t* pmasks, const float* in,
                 int n, int h, int wd)
{
    if (!d || !w || !in) return 1;
    if (d->c_out <= 0 || d->c_in <= 0 || n < 0 || h <= 0 || wd <= 0) return 1;
    if (d->stride < 1 || d->pad < 0) return 1;
    if (d->depthwise && d->c_in != d->c_out) return 1;
    if (!d->dense) {
        if (!ids || !pmasks || d->num_patterns <= 0) return 1;
        const size_t nk = (size_t)d->c_out * (d->depthwise ? 1 : d->c_in);
        for (size_t i = 0; i < nk; ++i)
            if ((!kmask || kmask[i]) && ids[i] >= d->num_patterns) return 2;
    }
    if (out_dim(h, d->pad, d->stride) <= 0 || out_dim(wd, d->pad, d->stride) <= 0) return 1;
    return 0;
}

/* Full output tensor, NCHW doubles.  Returns 0, 1 (bad argument) or 2 (pattern id
 * out of range). */
int patdnn_ref_conv2d(const patdnn_ref_desc* d, const float* w, const uint8_t* ids,
                      const uint8_t* kmask, const uint16_t* pmasks, const float* in,
                      int n, int h, int wd, const float* bias, double* out)
{
    int rc = check(d, w, ids, kmask, pmasks, in, n, h, wd);
    if (rc) return rc;
    if (!out) return 1;
    const int ho = out_dim(h, d->pad, d->stride), wo = out_dim(wd, d->pad, d->stride);
    const long planes = (long)n * d->c_out;
#ifdef _OPENMP
    if (d->nthreads > 0) omp_set_num_threads(d->nthreads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < planes; ++p) {
        const int img = (int)(p / d->c_out), co = (int)(p % d->c_out);
        double* o = out + (size_t)p * ho * wo;
        for (int oh = 0; oh < ho; ++oh)
            for (int ow = 0; ow < wo; ++ow)
                o[(size_t)oh * wo + ow] =
                    one_output(d, w, ids, kmask, pmasks, in, h, wd, bias, img, co, oh, ow);
    }
    return 0;
}

/* Selected output elements only: coords is [npts][4] = (n, co, oh, ow). */
int patdnn_ref_conv2d_points(const patdnn_ref_desc* d, const float* w, const uint8_t* ids,
                             const uint8_t* kmask, const uint16_t* pmasks, const float* in,
                             int n, int h, int wd, const float* bias,
                             const int32_t* coords, long npts, double* out)
{
    int rc = check(d, w, ids, kmask, pmasks, in, n, h, wd);
    if (rc) return rc;
    if (npts && (!coords || !out)) return 1;
    const int ho = out_dim(h, d->pad, d->stride), wo = out_dim(wd, d->pad, d->stride);
    for (long i = 0; i < npts; ++i) {
        const int32_t* c = coords + 4 * i;
        if (c[0] < 0 || c[0] >= n || c[1] < 0 || c[1] >= d->c_out ||
            c[2] < 0 || c[2] >= ho || c[3] < 0 || c[3] >= wo) return 1;
    }
#ifdef _OPENMP
    if (d->nthreads > 0) omp_set_num_threads(d->nthreads);
#endif
#pragma omp parallel for schedule(static)
    for (long i = 0; i < npts; ++i) {
        const int32_t* c = coords + 4 * i;
        out[i] = one_output(d, w, ids, kmask, pmasks, in, h, wd, bias, c[0], c[1], c[2], c[3]);
    }
    return 0;
}

int patdnn_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
