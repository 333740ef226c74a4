// Tiled pattern-sparse 3x3 convolution for gfx950 (wave64).
//
// Work decomposition
//   * The output is cut into "bands": PR output rows x (TGX*PC) output columns of one
//     image.  A wavefront covers NB = 64/TGX bands; lane (b, gx) owns a PR x PC patch of
//     outputs of band b, for all G filters of ONE filter group: G*PR*PC accumulators
//     in VGPRs.
//   * A workgroup is `waves` wavefronts that share the same NB bands and take
//     consecutive filter groups.  Input channels are staged through LDS, `ck`
//     channels at a time, band by band with a one-pixel halo, zero-filled outside
//     the image (the paper's input tiling, section 5.4).  Staging uses buffer loads
//     that write LDS directly (no registers; out-of-image lanes carry an out-of-range
//     offset and read as zero) into two alternating LDS buffers, so the loads of chunk
//     k+1 are in flight while chunk k is computed.
//   * Per staged channel a lane loads its (PR-1)*S+3 x (PC-1)*S+3 input window into
//     registers ONCE and applies every kept kernel of the group on that channel to
//     it: the window is reused across the taps and output rows of a kernel
//     (kernel-level load-redundancy elimination, section 5.4) and across the
//     filters of the group (filter-level elimination).
//   * The kept kernels of a group reach the wavefront as a record stream written by
//     the encoder ("load window of channel c", "kernel: slot, pattern, 4 weights",
//     "end of chunk").  A generated interpreter (gen_dispatch.py) reads it over the
//     scalar data path and jumps, per record, into a straight-line block of 4*PR*PC
//     FMAs with the weights as scalar operands - one generated body per pattern, no
//     indirect addressing, no per-lane branches (section 5.2 / 5.4).  The pattern
//     index ranges over the 56 centre-keeping patterns of section 4.1.
//   * Dense (unpruned) layers use the same staging and register tiling with a plain
//     9-tap loop and no stream.
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <mutex>
#include <type_traits>
#include <vector>

#include "kernels.hpp"
#include "layout.hpp"

namespace patdnn {

struct TiledArgs {
    const float* in;
    const float* bias;
    float* out;
    const int32_t* slot_channel;
    const uint32_t* chunk_ptr;
    const uint32_t* steps;
    const float* w9;
    int32_t n, c_in, c_out, h, w, ho, wo, pad, relu, pool;
    int32_t num_groups, bx, by, num_bands, ck, num_chunks, waves, fgsets;
    FastDiv div_bx, div_by, div_fgsets, div_bxby;   // for divisions by bx, by, fgsets and bx*by
    // issue priority (see the kernel): workgroups with a linear index >= late_from are in the
    // last round of the launch and run one level higher per late_span workgroups; late_span 0
    // with late_from 0 = the launch is a single round, priority follows the remaining work;
    // late_from INT32_MAX = every wavefront stays at the default priority
    int32_t late_from, late_span;
    // split launches: 0 = the slices ADD into `out` (zeroed beforehand) with atomics; otherwise
    // slice y STORES its partial sums to out + y * slice_stride (floats), a buffer of its own
    size_t slice_stride;
#ifdef PATDNN_TIMELINE
    unsigned long long* tl;      // [blocks][8 waves][8 phases] cycle totals (debug builds only)
#endif
};

// Phase timeline for performance work: a build with -DPATDNN_TIMELINE makes every wavefront add
// up the cycles it spends in each phase (prologue, waiting for staged data, issuing staging
// loads, the chunk's kernels, epilogue, barriers) and write the totals to the buffer given to
// patdnn_debug_timeline(): a tool for finding where a wavefront's time goes.  The product build
// does not define the macro and compiles none of it.
#ifdef PATDNN_TIMELINE
#define TL_DECL unsigned long long tl_t = __builtin_readcyclecounter(), tl_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define TL_MARK(k) do { const unsigned long long now = __builtin_readcyclecounter(); tl_acc[k] += now - tl_t; tl_t = now; } while (0)
#else
#define TL_DECL
#define TL_MARK(k)
#endif

template <int G_, int PR_, int PC_, int S_, int TGX_, bool DENSE_, int MAXSLOTS_, int MODE_>
struct Geo {
    static constexpr int G = G_, PR = PR_, PC = PC_, S = S_, TGX = TGX_, MAXSLOTS = MAXSLOTS_, MODE = MODE_;
    static constexpr bool DENSE = DENSE_;
    static constexpr int NB = 64 / TGX;                 // bands per wavefront
    static constexpr int WR = (PR - 1) * S + 3;         // window (= staged band) rows
    static constexpr int WC = (PC - 1) * S + 3;         // window columns per lane
    static constexpr int PITCH = (TGX * PC - 1) * S + 3;  // staged band columns
    // LDS layout of one staged channel.
    // Row-interleaved (MODE bit 3 clear): [window row][band][column] - the same row of the
    // NB bands side by side, so that 64 consecutive LDS dwords (what one staging
    // instruction of a wavefront fills) come from a short run of one image row when the
    // bands are neighbours in x.
    // Band-major (MODE bit 3 set): [band][window row][column], bands BANDP floats apart
    // with BANDP = lanes-per-band step (mod 32), so that the lanes of half a wavefront
    // fall on 32 different LDS banks when they read the same window element.
    static constexpr bool BAND_MAJOR = (MODE & 8) != 0;
    static constexpr int ROWP = NB * PITCH;             // floats per staged row (row-interleaved)
    static constexpr int BAND = WR * PITCH;             // floats of one band
    static constexpr int BANDP = BAND + ((TGX * PC * S) % 32 - BAND % 32 + 32) % 32;
    static constexpr int RSTRIDE = BAND_MAJOR ? PITCH : ROWP;    // between a lane's window rows
    static constexpr int BSTRIDE = BAND_MAJOR ? BANDP : PITCH;   // between bands
    // floats per staged channel; a multiple of 64 (one staging instruction = 64 dwords)
    static constexpr int TILEP = ((BAND_MAJOR ? NB * BANDP : WR * ROWP) + 63) / 64 * 64;
    static constexpr int NACC = PR * PC;
};

// StreamLoop<G,PR,PC,S,TGX,MODE>::run(acc, lane_lds, stream, entry): the step interpreter
// with its table of pattern-specialised FMA blocks (gen_dispatch.py).
template <int G, int PR, int PC, int S, int TGX, int MODE>
struct StreamLoop;

// dense variants have no stream
template <int G, int PR, int PC, int S, int TGX, int MODE>
struct NoStream {
    static constexpr unsigned kBlockBytes = 0, kTableOff = 0, kCtrlBytes = 0, kRecords = 0;
};

#include "gen/dispatch_all.inc"

// Wave-uniform read-only data (layer metadata, weights) is fetched through the
// constant address space so that it travels over the scalar data path into SGPRs.
template <class T>
__device__ __forceinline__ T load_uniform(const T* p, size_t i)
{
    typedef const T __attribute__((address_space(4))) * cptr;
    return ((cptr)(uintptr_t)p)[i];
}

typedef __attribute__((address_space(3))) float lds_f32;

// SPLITK: the workgroup covers only the chunks [chunk_first, chunk_last) of the input
// channels and ADDS its partial sums to the output (which the launcher zeroed; bias and
// ReLU are applied by a finishing kernel): more workgroups for layers with few tiles.
// blockIdx.y = slice of the input channels: chunks [y*n/k, (y+1)*n/k), k = gridDim.y.
template <class GEO, bool SPLITK>
__global__ __launch_bounds__(512) void tiled_conv_kernel(TiledArgs a)
{
    constexpr int G = GEO::G, PR = GEO::PR, PC = GEO::PC, S = GEO::S, TGX = GEO::TGX;
    constexpr int NB = GEO::NB, WR = GEO::WR, WC = GEO::WC, PITCH = GEO::PITCH;
    extern __shared__ float lds[];
    TL_DECL;

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups are handed to the 8 XCDs round-robin by blockIdx; renumber them so that
    // each XCD works on a contiguous range: the workgroups that stage the same bands
    // (different filter groups) then share one L2.
    const int nblk = gridDim.x;
    const int per_xcd = nblk >> 3, xcd = blockIdx.x & 7, rank = blockIdx.x >> 3;
    const int bid = rank < per_xcd ? xcd * per_xcd + rank : blockIdx.x;   // tail (< 8 blocks) keeps its id
    const int tile = (int)fast_div((uint32_t)bid, a.div_fgsets);
    const int fgset = bid - tile * a.fgsets;
    const int group = fgset * a.waves + wave;
    const int band0 = tile * NB;
    const int plane = a.h * a.w;

    // image of the tile's first band: staging offsets are relative to it
    const int img0 = (int)fast_div((uint32_t)band0, a.div_bxby);
    const float* in_blk = a.in + (size_t)img0 * a.c_in * plane;

    // ---- staging slots of this thread: byte offset (inside the tile's first image
    // onwards) of the input element that lands in LDS dword tid + k*nthreads of a staged
    // channel; ~0u (out of range for the buffer descriptor, reads as zero) for padding
    unsigned voff[GEO::MAXSLOTS];
#pragma unroll
    for (int k = 0; k < GEO::MAXSLOTS; ++k) {
        const int e = tid + k * nthreads;
        voff[k] = ~0u;
        int q, b, x;
        if constexpr (GEO::BAND_MAJOR) {
            b = e / GEO::BANDP;
            const int rem = e - b * GEO::BANDP;
            q = rem / PITCH;
            x = rem - q * PITCH;
            if (b >= NB) q = WR;                        // beyond the last band: padding
        } else {
            q = e / GEO::ROWP;
            const int rem = e - q * GEO::ROWP;
            b = rem / PITCH;
            x = rem - b * PITCH;
        }
        if (q < WR) {
            const int band = band0 + b;
            if (band < a.num_bands) {
                const int t = (int)fast_div((uint32_t)band, a.div_bx), bxi = band - t * a.bx;
                const int img = (int)fast_div((uint32_t)t, a.div_by), byi = t - img * a.by;
                const int iy = byi * PR * S - a.pad + q;
                const int ix = bxi * TGX * PC * S - a.pad + x;
                if (iy >= 0 && iy < a.h && ix >= 0 && ix < a.w)
                    voff[k] = 4u * (unsigned)((img - img0) * a.c_in * plane + iy * a.w + ix);
            }
        }
    }
    // bytes from the tile's first image to the end of the input tensor
    const size_t blk_bytes = (size_t)(a.n - img0) * a.c_in * plane * 4;
    lds_f32* const lds3 = (lds_f32*)lds;
    const int buf_floats = a.ck * GEO::TILEP;

    // Staging instructions of this wavefront per channel: slot k fills LDS dwords
    // [wave*64 + k*nthreads, +64) of the channel, so the count is the same for every channel
    // and the per-channel code is straight-line (a taken branch costs about as much as ten
    // loads take to issue).
    const int my_slots = __builtin_amdgcn_readfirstlane(
        max(0, min((int)GEO::MAXSLOTS, (GEO::TILEP - wave * 64 + nthreads - 1) / nthreads)));
    auto stage_n = [&](auto nk_tag, int c0, lds_f32* buf) __attribute__((always_inline)) {
        constexpr int NK = decltype(nk_tag)::value;
        const int cn = min(a.ck, a.c_in - c0);
        const char* src = (const char*)in_blk + (size_t)c0 * plane * 4;
        size_t left = blk_bytes - (size_t)c0 * plane * 4;
        lds_f32* dst = buf + wave * 64;
        for (int c = 0; c < cn; ++c) {
            const unsigned nrec = left > 0xFFFFFFFFull ? 0xFFFFFFFFu : (unsigned)left;
            __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)src, 0, (int)nrec, 0x00020000);
#pragma unroll
            for (int k = 0; k < NK; ++k)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst + k * nthreads, 4, (int)voff[k], 0, 0, 0);
            src += (size_t)plane * 4;
            left -= (size_t)plane * 4;
            dst += GEO::TILEP;
        }
    };
    auto stage = [&](int c0, lds_f32* buf) __attribute__((always_inline)) {
        static_assert(GEO::MAXSLOTS <= 16, "staging slots per thread");
        switch (my_slots) {
#define PATDNN_STAGE_CASE(n) case n: if constexpr (n <= GEO::MAXSLOTS) stage_n(std::integral_constant<int, n>{}, c0, buf); break;
            PATDNN_STAGE_CASE(1) PATDNN_STAGE_CASE(2) PATDNN_STAGE_CASE(3) PATDNN_STAGE_CASE(4)
            PATDNN_STAGE_CASE(5) PATDNN_STAGE_CASE(6) PATDNN_STAGE_CASE(7) PATDNN_STAGE_CASE(8)
            PATDNN_STAGE_CASE(9) PATDNN_STAGE_CASE(10) PATDNN_STAGE_CASE(11) PATDNN_STAGE_CASE(12)
            PATDNN_STAGE_CASE(13) PATDNN_STAGE_CASE(14) PATDNN_STAGE_CASE(15) PATDNN_STAGE_CASE(16)
#undef PATDNN_STAGE_CASE
            default: break;
        }
    };

    // ---- this lane's patch
    const int lb = lane / TGX, gx = lane - lb * TGX;
    const int my_band = band0 + lb;
    // when TGX does not divide 64 the last lanes of the wavefront have no band
    const bool lane_ok = (64 % TGX == 0) || lb < NB;
    const bool band_ok = lane_ok && my_band < a.num_bands;
    int img = 0, oy0 = 0, ox0 = 0;
    if (band_ok) {
        const int t = (int)fast_div((uint32_t)my_band, a.div_bx), bxi = my_band - t * a.bx;
        img = (int)fast_div((uint32_t)t, a.div_by);
        const int byi = t - img * a.by;
        oy0 = byi * PR;
        ox0 = (bxi * TGX + gx) * PC;
    }
    const int lane_off = lane_ok ? lb * GEO::BSTRIDE + gx * PC * S : 0;   // floats, inside one staged channel

    float acc[G][GEO::NACC];
#pragma unroll
    for (int s = 0; s < G; ++s)
#pragma unroll
        for (int i = 0; i < GEO::NACC; ++i) acc[s][i] = 0.0f;

    const bool group_ok = group < a.num_groups;

    int chunk_first = 0, c_first = 0, c_end = a.c_in, chunks_here = a.num_chunks;
    if constexpr (SPLITK) {
        const int k = (int)gridDim.y, y = (int)blockIdx.y;
        chunk_first = (int)((long long)a.num_chunks * y / k);
        const int chunk_last = (int)((long long)a.num_chunks * (y + 1) / k);
        chunks_here = chunk_last - chunk_first;
        c_first = chunk_first * a.ck;
        c_end = min(a.c_in, chunk_last * a.ck);
    }
    // MODE bit 4: ONE staging buffer (half the LDS, so twice the channels per chunk or more
    // workgroups per CU); the chunk is loaded after everyone has left the previous one and
    // the other workgroups of the CU cover the wait.  Otherwise two alternating buffers.
    constexpr bool ONE_BUFFER = (GEO::MODE & 16) != 0;
    // ---- issue priority.  A SIMD serves its oldest wavefront first, so the wavefronts that
    // start last (the last round of workgroups, dispatched as the earlier ones retire) crawl
    // behind their older neighbours and then finish alone, at a third of the SIMD's rate: the
    // launch ends one lonely wavefront life after the machine has run out of work.  The
    // workgroups of the last round therefore issue at raised priority, the later dispatched
    // the higher (levels 1..3 over the round), and the launch ends close to the time its
    // last-dispatched workgroup needs on its own.  A launch of a single round has no late
    // workgroups; there the priority follows the remaining work (set per chunk below), so that
    // the wavefronts sharing a SIMD finish together instead of one after the other.
    const int late = (int)(blockIdx.y * gridDim.x + blockIdx.x) - a.late_from;
    if (late >= 0 && a.late_span > 0) {
        const int level = late / a.late_span;
        if (level == 0) __builtin_amdgcn_s_setprio(1);
        else if (level == 1) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(3);
    }
    TL_MARK(0);                                   // prologue
    if constexpr (!ONE_BUFFER) stage(c_first, lds3);
    TL_MARK(2);
    for (int c0 = c_first, chunk = SPLITK ? chunk_first : 0; c0 < c_end; c0 += a.ck, ++chunk) {
        const int cn = min(a.ck, a.c_in - c0);
        const int cur = ONE_BUFFER ? 0 : ((SPLITK ? chunk - chunk_first : chunk) & 1) * buf_floats;
        if (a.late_span == 0 && a.late_from == 0) {
            // single round: the wavefronts that are behind issue first (quarters of the
            // slice's chunks, by comparison: no division in the loop)
            const int done4 = 4 * (chunk - (SPLITK ? chunk_first : 0));
            if (done4 < chunks_here) __builtin_amdgcn_s_setprio(3);
            else if (done4 < 2 * chunks_here) __builtin_amdgcn_s_setprio(2);
            else if (done4 < 3 * chunks_here) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        if constexpr (ONE_BUFFER) {
            __syncthreads();                      // everyone has finished reading the buffer
            TL_MARK(5);                           // barrier
            stage(c0, lds3);
            TL_MARK(2);                           // issuing the chunk's loads
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
            TL_MARK(1);                           // wait for the staged chunk
            __syncthreads();
            TL_MARK(6);                           // second barrier
        } else {
            // chunk `chunk` has landed in this wavefront's view, and (barrier) in everyone's;
            // everyone has also finished reading the other buffer
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
            TL_MARK(1);                           // wait for the staged chunk
            __syncthreads();
            TL_MARK(5);                           // barrier
            if (c0 + a.ck < c_end) stage(c0 + a.ck, lds3 + (buf_floats - cur));
            TL_MARK(2);                           // issuing the next chunk's loads
        }

        if (group_ok) {
            if constexpr (GEO::DENSE) {
                for (int c = 0; c < cn; ++c) {
                    float win[WR * WC];
                    const float* base = lds + cur + lane_off + c * GEO::TILEP;
#pragma unroll
                    for (int q = 0; q < WR; ++q)
#pragma unroll
                        for (int r = 0; r < WC; ++r) win[q * WC + r] = base[q * GEO::RSTRIDE + r];
                    const float* wp = a.w9 + ((size_t)group * a.c_in + (c0 + c)) * (G * 9);
#pragma unroll
                    for (int s = 0; s < G; ++s)
#pragma unroll
                        for (int pos = 0; pos < 9; ++pos) {
                            const float wv = load_uniform(wp, s * 9 + pos);
#pragma unroll
                            for (int r = 0; r < PR; ++r)
#pragma unroll
                                for (int cc = 0; cc < PC; ++cc)
                                    acc[s][r * PC + cc] =
                                        fmaf(wv, win[(r * S + pos / 3) * WC + cc * S + pos % 3],
                                             acc[s][r * PC + cc]);
                        }
                }
            } else {
                // the group's steps of this chunk: first step, and (threaded dispatch) the
                // control block that enters it
                const unsigned cp = load_uniform(a.chunk_ptr, (size_t)group * a.num_chunks + chunk);
                const unsigned start = cp & kChunkStepMask;
                using Loop = StreamLoop<G, PR, PC, S, TGX, (GEO::MODE & 15)>;   // bit 4 is the kernel's, not the interpreter's
                const unsigned lds_base =
                    (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)lds;
                Loop::run(acc, lds_base + 4u * (unsigned)(cur + lane_off),
                          a.steps + (size_t)start * kStepDwords, (cp >> kChunkEntryShift) * Loop::kCtrlBytes);
            }
        }
        TL_MARK(3);                               // the chunk's kernels
    }

    // ---- epilogue: bias, ReLU, scatter to the original output channel
    // A split launch either adds its slices up in the output with atomics, or (slice_stride != 0)
    // gives every slice a buffer of its own, which it fills with the plain stores of the unsplit
    // epilogue (bias NULL, no activation: the launcher sees to both); a finishing kernel adds the
    // buffers up in a fixed order.
    const bool to_slices = SPLITK && a.slice_stride != 0;
    float* const out_base = SPLITK ? a.out + (size_t)blockIdx.y * a.slice_stride : a.out;
    bool written = false;
    if constexpr (SPLITK && PC == 2 && 64 % (TGX * PC) == 0) {
      if (!to_slices) {
        written = true;
        // Partial sums go out as atomic adds, which run at full rate only on whole runs of
        // consecutive floats: 16 lanes on 16 neighbouring outputs cost next to nothing, the
        // same values written lane by lane (a lane's two outputs of a row are neighbours, so
        // one instruction touches every second float of its lines) cost 0.15 ms per 25 MB.
        // The lanes therefore trade values first: instruction h = 0, 1 of a row covers the
        // rows of half the wavefront's bands, TGX*PC consecutive lanes per band row, each lane
        // taking its column from the lane that accumulated it.  The exchange runs with every
        // lane of the wavefront (outside the per-lane conditions); only the atomics are
        // predicated.
        if (group_ok) {
            constexpr int BW = TGX * PC;                 // columns of a band row
            constexpr int BPI = 64 / BW;                 // band rows per instruction
            const size_t oplane = (size_t)a.ho * a.wo;
            int src[2], rows_left[2];
            bool odd[2], ok[2];
            size_t off[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int tb = h * BPI + lane / BW;      // band of the wavefront this lane writes
                const int col = lane - (lane / BW) * BW;
                const int owner = (tb * TGX) << 2;       // its first lane: ox0 there is the band's first column
                const int t_img = __builtin_amdgcn_ds_bpermute(owner, img);
                const int t_oy0 = __builtin_amdgcn_ds_bpermute(owner, oy0);
                const int t_x0 = __builtin_amdgcn_ds_bpermute(owner, ox0);
                const int t_ok = __builtin_amdgcn_ds_bpermute(owner, band_ok ? 1 : 0);
                src[h] = owner + ((col >> 1) << 2);
                odd[h] = (col & 1) != 0;
                ok[h] = t_ok != 0 && t_x0 + col < a.wo;
                rows_left[h] = a.ho - t_oy0;
                off[h] = ((size_t)t_img * a.c_out * a.ho + t_oy0) * (size_t)a.wo + t_x0 + col;
            }
#pragma unroll
            for (int s = 0; s < G; ++s) {
                const int co = load_uniform(a.slot_channel, group * G + s);
                if (co < 0) continue;
                float* dst = a.out + (size_t)co * oplane;
#pragma unroll
                for (int r = 0; r < PR; ++r) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const float even = __int_as_float(__builtin_amdgcn_ds_bpermute(src[h], __float_as_int(acc[s][r * PC])));
                        const float oddv = __int_as_float(__builtin_amdgcn_ds_bpermute(src[h], __float_as_int(acc[s][r * PC + 1])));
                        if (ok[h] && r < rows_left[h]) unsafeAtomicAdd(&dst[off[h] + (size_t)r * a.wo], odd[h] ? oddv : even);
                    }
                }
            }
        }
      }
    }
    if (!written && group_ok && band_ok) {
        const size_t oplane = (size_t)a.ho * a.wo;
        if (!SPLITK && a.pool && PC == 2) {
            // ReLU + 2x2 max pooling with two columns per lane: a lane's columns are the two
            // columns of one pooled column (ox0 is even), and of its PR rows all but one pair up
            // inside the patch, so most pooled cells are complete in registers and go out as
            // plain stores; only the row whose partner belongs to the band above or below (the
            // first row where the band starts at an odd row, else the last) is folded into its
            // zeroed cell with the atomic max, like the values of the general path below.
            const int pho = a.ho >> 1, pwo = a.wo >> 1;
            const int px = ox0 >> 1;
            const bool odd_start = (oy0 & 1) != 0;
#pragma unroll
            for (int s = 0; s < G; ++s) {
                const int co = load_uniform(a.slot_channel, group * G + s);
                if (co < 0) continue;
                const float b = a.bias ? load_uniform(a.bias, co) : 0.0f;
                float* dstf = a.out + ((size_t)img * a.c_out + co) * ((size_t)pho * pwo);
                unsigned* dst = reinterpret_cast<unsigned*>(dstf);
                float m[PR];                     // max over the lane's two columns, ReLU applied
#pragma unroll
                for (int r = 0; r < PR; ++r) m[r] = fmaxf(fmaxf(acc[s][r * PC], acc[s][r * PC + 1]) + b, 0.0f);
                if (px < pwo) {
#pragma unroll
                    for (int r = 0; r + 1 < PR; ++r) {
                        // rows r, r + 1 form a window if the upper one is an even row of the image
                        const int oy = oy0 + r;
                        if (((r & 1) != 0) == odd_start && (oy >> 1) < pho)
                            dstf[(size_t)(oy >> 1) * pwo + px] = fmaxf(m[r], m[r + 1]);
                    }
                    // the row left over: 0 for a band that starts at an odd row, else the last one
                    // if the patch has an odd number of rows
                    if (odd_start) {
                        if (m[0] > 0.0f && (oy0 >> 1) < pho) atomicMax(&dst[(size_t)(oy0 >> 1) * pwo + px], __float_as_uint(m[0]));
                    }
                    if (((PR & 1) != 0) != odd_start) {
                        const int oy = oy0 + PR - 1;
                        if (m[PR - 1] > 0.0f && (oy >> 1) < pho)
                            atomicMax(&dst[(size_t)(oy >> 1) * pwo + px], __float_as_uint(m[PR - 1]));
                    }
                }
            }
        } else if (!SPLITK && a.pool) {
            // ReLU + 2x2 max pooling: fold every value into its pooled cell (zero beforehand)
            const int pho = a.ho >> 1, pwo = a.wo >> 1;
#pragma unroll
            for (int s = 0; s < G; ++s) {
                const int co = load_uniform(a.slot_channel, group * G + s);
                if (co < 0) continue;
                const float b = a.bias ? load_uniform(a.bias, co) : 0.0f;
                unsigned* dst = reinterpret_cast<unsigned*>(a.out) + ((size_t)img * a.c_out + co) * ((size_t)pho * pwo);
#pragma unroll
                for (int r = 0; r < PR; ++r)
#pragma unroll
                    for (int c = 0; c < PC; ++c) {
                        const int oy = oy0 + r, ox = ox0 + c;
                        const float v = acc[s][r * PC + c] + b;
                        if (v > 0.0f && (oy >> 1) < pho && (ox >> 1) < pwo)
                            atomicMax(&dst[(size_t)(oy >> 1) * pwo + (ox >> 1)], __float_as_uint(v));
                    }
            }
        } else if ((!SPLITK || to_slices) && PC == 2 && (a.wo & 1) == 0 && (reinterpret_cast<uintptr_t>(out_base) & 7) == 0) {
            // a lane's two outputs of a row are neighbours at an even column: with an even row
            // length (and an 8-byte aligned tensor) they go out as one 8-byte store
            struct alignas(8) Pair { float x, y; };
#pragma unroll
            for (int s = 0; s < G; ++s) {
                const int co = load_uniform(a.slot_channel, group * G + s);
                if (co < 0) continue;
                const float b = a.bias ? load_uniform(a.bias, co) : 0.0f;
                float* dst = out_base + ((size_t)img * a.c_out + co) * oplane;
#pragma unroll
                for (int r = 0; r < PR; ++r) {
                    const int oy = oy0 + r;
                    Pair v{acc[s][r * PC] + b, acc[s][r * PC + 1] + b};
                    if (a.relu) { v.x = fmaxf(v.x, 0.0f); v.y = fmaxf(v.y, 0.0f); }
                    if (oy < a.ho && ox0 < a.wo) *reinterpret_cast<Pair*>(&dst[(size_t)oy * a.wo + ox0]) = v;
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < G; ++s) {
                const int co = load_uniform(a.slot_channel, group * G + s);
                if (co < 0) continue;
                const float b = a.bias ? load_uniform(a.bias, co) : 0.0f;
                float* dst = out_base + ((size_t)img * a.c_out + co) * oplane;
#pragma unroll
                for (int r = 0; r < PR; ++r)
#pragma unroll
                    for (int c = 0; c < PC; ++c) {
                        const int oy = oy0 + r, ox = ox0 + c;
                        if (SPLITK && !to_slices) {
                            if (oy < a.ho && ox < a.wo) unsafeAtomicAdd(&dst[(size_t)oy * a.wo + ox], acc[s][r * PC + c]);
                        } else {
                            float v = acc[s][r * PC + c] + b;
                            if (a.relu) v = fmaxf(v, 0.0f);
                            if (oy < a.ho && ox < a.wo) dst[(size_t)oy * a.wo + ox] = v;
                        }
                    }
            }
        }
    }
#ifdef PATDNN_TIMELINE
    TL_MARK(4);                                   // epilogue (stores issued)
    if (a.tl && lane == 0)
        for (int k = 0; k < 8; ++k) a.tl[((size_t)blockIdx.x * 8 + wave) * 8 + k] = tl_acc[k];
#endif
}

#ifdef PATDNN_TIMELINE
static unsigned long long* g_timeline = nullptr;
extern "C" void patdnn_debug_timeline(unsigned long long* p) { g_timeline = p; }
#endif

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.0f;
}

// out[n][c][pixel] = act(sum + bias[c]) after a split launch: `sum` is the output itself (the
// slices were added up in place with atomics; slices == 1) or `slices` buffers of partial sums,
// slice_stride floats apart, added here in the order of the slices.
// A unit is VEC floats of one plane (VEC = 4 where planes are whole aligned float4s); which
// channel a unit belongs to comes from multiplications where the count allows (a 64-bit
// division per element would cost more than the memory traffic of a small layer).
struct FinishArgs {
    float* zero;                         // also cleared by this launch (the next launch's target), or NULL
    size_t zero_count;
    size_t plane_units, total_units;
    FastDiv div_plane, div_c;            // used when total_units < 2^31
    int c_out, relu;
    const float* sums;                   // first buffer of partial sums (== out when added in place)
    size_t slice_stride;                 // floats between the buffers
    int slices;
};

template <int VEC>
__global__ __launch_bounds__(256) void bias_act_kernel(float* out, const float* bias, FinishArgs a)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const bool small = a.total_units <= 0x7FFFFFFFull;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.zero_count; i += stride) a.zero[i] = 0.0f;
    for (size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x; u < a.total_units; u += stride) {
        float b = 0.0f;
        if (bias) {
            size_t c;
            if (small) {
                const uint32_t pl = fast_div((uint32_t)u, a.div_plane);
                c = pl - fast_div(pl, a.div_c) * (uint32_t)a.c_out;
            } else {
                c = (u / a.plane_units) % (size_t)a.c_out;
            }
            b = bias[c];
        }
        if constexpr (VEC == 4) {
            // up to eight buffers' loads in flight at a time (a single image splits into up to 32
            // slices; one load after the other would cost their latencies in a row); the
            // additions stay in slice order
            auto part = [&](int k) { return reinterpret_cast<const float4*>(a.sums + (size_t)k * a.slice_stride)[u]; };
            float4 v = part(0);
            int k = 1;
            for (; k + 7 < a.slices; k += 8) {
                float4 t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t[j] = part(k + j);
#pragma unroll
                for (int j = 0; j < 8; ++j) { v.x += t[j].x; v.y += t[j].y; v.z += t[j].z; v.w += t[j].w; }
            }
            for (; k + 3 < a.slices; k += 4) {
                const float4 t0 = part(k), t1 = part(k + 1), t2 = part(k + 2), t3 = part(k + 3);
                v.x += t0.x; v.y += t0.y; v.z += t0.z; v.w += t0.w;
                v.x += t1.x; v.y += t1.y; v.z += t1.z; v.w += t1.w;
                v.x += t2.x; v.y += t2.y; v.z += t2.z; v.w += t2.w;
                v.x += t3.x; v.y += t3.y; v.z += t3.z; v.w += t3.w;
            }
            for (; k < a.slices; ++k) {
                const float4 t = part(k);
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            }
            v.x += b; v.y += b; v.z += b; v.w += b;
            if (a.relu) { v.x = fmaxf(v.x, 0.0f); v.y = fmaxf(v.y, 0.0f); v.z = fmaxf(v.z, 0.0f); v.w = fmaxf(v.w, 0.0f); }
            reinterpret_cast<float4*>(out)[u] = v;
        } else {
            float v = a.sums[u];
            int k = 1;
            for (; k + 3 < a.slices; k += 4) {
                const float t0 = a.sums[(size_t)k * a.slice_stride + u], t1 = a.sums[(size_t)(k + 1) * a.slice_stride + u];
                const float t2 = a.sums[(size_t)(k + 2) * a.slice_stride + u], t3 = a.sums[(size_t)(k + 3) * a.slice_stride + u];
                v += t0; v += t1; v += t2; v += t3;
            }
            for (; k < a.slices; ++k) v += a.sums[(size_t)k * a.slice_stride + u];
            v += b;
            if (a.relu) v = fmaxf(v, 0.0f);
            out[u] = v;
        }
    }
}

static void launch_bias_act(float* out, const float* sums, int slices, size_t slice_stride, const float* bias,
                            int c_out, size_t plane, size_t total, int relu, float* zero, size_t zero_count,
                            hipStream_t stream)
{
    const bool vec = plane % 4 == 0 && ((reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(sums)) & 15) == 0 &&
                     slice_stride % 4 == 0;
    FinishArgs a{};
    a.sums = sums;
    a.slices = slices;
    a.slice_stride = slice_stride;
    a.zero = zero;
    a.zero_count = zero ? zero_count : 0;
    a.plane_units = vec ? plane / 4 : plane;
    a.total_units = vec ? total / 4 : total;
    a.div_plane = make_fast_div((uint32_t)std::min<size_t>(a.plane_units, 0x7FFFFFFFu));
    a.div_c = make_fast_div((uint32_t)c_out);
    a.c_out = c_out;
    a.relu = relu;
    const unsigned blocks = (unsigned)std::min<size_t>((std::max(a.total_units, a.zero_count / 4) + 255) / 256, 256 * 32);
    if (blocks == 0) return;
    if (vec) hipLaunchKernelGGL(bias_act_kernel<4>, dim3(blocks), dim3(256), 0, stream, out, bias, a);
    else hipLaunchKernelGGL(bias_act_kernel<1>, dim3(blocks), dim3(256), 0, stream, out, bias, a);
}

// More than 64 KB of dynamic LDS needs the function attribute, once per device (bit = device
// id); two threads racing here both set it, which is harmless.
static hipError_t allow_big_lds(const void* fn, std::atomic<uint64_t>& done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// out[n][c][py][px] = max over the 2x2 window of relu(sum[n][c][2py+dy][2px+dx] + bias[c]):
// finishes a split-channel launch whose partial sums were added up in `sum` (slices == 1) or
// lie in `slices` buffers, slice_stride floats apart, from `sum` on
__global__ __launch_bounds__(256) void bias_relu_pool_kernel(const float* sum, const float* bias, float* out,
                                                             int c_out, int ho, int wo, int pho, int pwo, size_t total,
                                                             FastDiv div_pwo, FastDiv div_pho, FastDiv div_c,
                                                             float* zero, size_t zero_count, int slices,
                                                             size_t slice_stride)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const bool small = total <= 0x7FFFFFFFull;      // then the divisions are multiplications
    // the next launch's target, cleared here to save it a launch (never the sums read below)
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < zero_count; i += stride) zero[i] = 0.0f;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int px, py;
        size_t r, c;                                // r = n * c_out + c
        if (small) {
            const uint32_t r1 = fast_div((uint32_t)i, div_pwo);
            px = (int)((uint32_t)i - r1 * (uint32_t)pwo);
            const uint32_t r2 = fast_div(r1, div_pho);
            py = (int)(r1 - r2 * (uint32_t)pho);
            r = r2;
            c = r2 - fast_div(r2, div_c) * (uint32_t)c_out;
        } else {
            px = (int)(i % pwo);
            r = i / pwo;
            py = (int)(r % pho);
            r /= pho;
            c = r % (size_t)c_out;
        }
        const float b = bias ? bias[c] : 0.0f;
        const float* src = sum + (r * ho + 2 * py) * (size_t)wo + 2 * px;
        float v00 = src[0], v01 = src[1], v10 = src[wo], v11 = src[wo + 1];
        for (int k = 1; k < slices; ++k) {           // buffers of partial sums, in slice order
            const float* t = src + (size_t)k * slice_stride;
            v00 += t[0]; v01 += t[1]; v10 += t[wo]; v11 += t[wo + 1];
        }
        const float m = fmaxf(fmaxf(v00, v01), fmaxf(v10, v11));
        out[i] = fmaxf(m + b, 0.0f);
    }
}

// Workgroups of `fn` that the current device holds at once with this block size and dynamic
// LDS (0 if the runtime cannot say).  Asked once per (device, kernel, block size, LDS size).
static long long resident_workgroups(const void* fn, int threads, size_t lds_bytes)
{
    struct Entry { int dev; const void* fn; int threads; size_t lds; long long slots; };
    static std::mutex lock;
    static std::vector<Entry> known;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    std::lock_guard<std::mutex> guard(lock);
    for (const Entry& e : known)
        if (e.dev == dev && e.fn == fn && e.threads == threads && e.lds == lds_bytes) return e.slots;
    int per_cu = 0, cus = 0;
    long long slots = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, threads, lds_bytes) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
        slots = (long long)per_cu * cus;
    known.push_back(Entry{dev, fn, threads, lds_bytes, slots});
    return slots;
}

// PATDNN_WAVE_PRIORITY=0 in the environment leaves every wavefront at the default priority
// (for measuring what the priorities buy); read once.
static bool wave_priority_enabled()
{
    static const bool on = [] {
        const char* e = std::getenv("PATDNN_WAVE_PRIORITY");
        return !(e && e[0] == '0' && e[1] == 0);
    }();
    return on;
}

template <class GEO>
static hipError_t launch_tiled(const DevTiled& t, const ConvShape& s, const float* in,
                               const float* bias, float* out, int32_t waves, int32_t ksplit,
                               float* scratch, size_t scratch_floats, hipStream_t stream)
{
    TiledArgs a{};
    a.in = in; a.bias = bias; a.out = out;
    a.slot_channel = t.slot_channel; a.chunk_ptr = t.chunk_ptr; a.steps = t.steps;
    a.w9 = t.w9;
    a.n = s.n; a.c_in = s.c_in; a.c_out = s.c_out; a.h = s.h; a.w = s.w; a.ho = s.ho; a.wo = s.wo;
    a.pad = s.pad; a.relu = s.relu; a.pool = s.pool;
    a.num_groups = t.num_groups;
    a.bx = (s.wo + GEO::TGX * GEO::PC - 1) / (GEO::TGX * GEO::PC);
    a.by = (s.ho + GEO::PR - 1) / GEO::PR;
    a.div_bx = make_fast_div((uint32_t)a.bx);
    a.div_by = make_fast_div((uint32_t)a.by);
    a.div_bxby = make_fast_div((uint32_t)a.bx * (uint32_t)a.by);
    const long long bands = (long long)s.n * a.bx * a.by;
    const long long tiles = (bands + GEO::NB - 1) / GEO::NB;
    a.num_bands = (int32_t)bands;
    a.ck = t.ck; a.num_chunks = t.num_chunks; a.waves = waves;
    a.fgsets = (t.num_groups + waves - 1) / waves;
    a.div_fgsets = make_fast_div((uint32_t)a.fgsets);
#ifdef PATDNN_TIMELINE
    a.tl = g_timeline;
#endif
    const long long blocks = tiles * a.fgsets;
    if (bands > INT32_MAX || blocks > INT32_MAX) return hipErrorInvalidValue;
    // every dword of a staged channel needs a staging slot of some thread
    if ((long long)waves * 64 * GEO::MAXSLOTS < GEO::TILEP || waves < 1 || waves > 8) return hipErrorInvalidValue;
    const size_t lds_bytes = ((GEO::MODE & 16) ? 1 : 2) * (size_t)t.ck * GEO::TILEP * sizeof(float);   // staging buffers
    if (lds_bytes > 64 * 1024) {
        static std::atomic<uint64_t> allowed{0};
        hipError_t e = allow_big_lds(reinterpret_cast<const void*>(&tiled_conv_kernel<GEO, false>), allowed);
        if (e != hipSuccess) return e;
    }
    // issue priorities from the workgroups of this launch that are resident at once (asked
    // after the kernel has been allowed its dynamic LDS: the answer depends on it)
    auto set_priorities = [&](const void* fn, long long all) {
        const long long slots = wave_priority_enabled() ? resident_workgroups(fn, 64 * waves, lds_bytes) : 0;
        a.late_from = INT32_MAX;
        a.late_span = 0;
        if (slots <= 0) return;
        if (all <= slots) {
            // a single round: by remaining work - where wavefronts share SIMDs at all
            if (2 * all > slots) a.late_from = 0;
        } else {
            a.late_from = (int32_t)(all - slots);
            a.late_span = (int32_t)((slots + 2) / 3);
        }
    };
    if (s.pool && ksplit > 1 && !scratch) return hipErrorInvalidValue;   // the slices need somewhere to add up
    if (ksplit <= 1) {
        set_priorities(reinterpret_cast<const void*>(&tiled_conv_kernel<GEO, false>), blocks);
        hipLaunchKernelGGL((tiled_conv_kernel<GEO, false>), dim3((unsigned)blocks), dim3(64 * waves), lds_bytes,
                           stream, a);
        return hipGetLastError();
    }
    // split over the input channels: zero the output, add the slices up, then bias + ReLU
    if constexpr (GEO::DENSE) {
        return hipErrorInvalidValue;
    } else {
        if (ksplit > t.num_chunks || ksplit > 65535) return hipErrorInvalidValue;
        if (lds_bytes > 64 * 1024) {
            static std::atomic<uint64_t> allowed_k{0};
            hipError_t e = allow_big_lds(reinterpret_cast<const void*>(&tiled_conv_kernel<GEO, true>), allowed_k);
            if (e != hipSuccess) return e;
        }
        set_priorities(reinterpret_cast<const void*>(&tiled_conv_kernel<GEO, true>), blocks * ksplit);
        const size_t plane = (size_t)s.ho * s.wo, total = (size_t)s.n * s.c_out * plane;
        const unsigned fill_blocks = (unsigned)std::min<size_t>((total + 255) / 256, 256 * 32);
        // With room for one buffer per slice the slices store their partial sums (no zero fill,
        // no atomics, and a sum in a fixed order: results repeat bit for bit); otherwise they add
        // into the output - or, for a pooled layer, into the one buffer there is room for.
        const size_t slice_stride = split_slice_stride(total);
        const bool to_slices = scratch && scratch_floats / (size_t)ksplit >= slice_stride &&
                               (reinterpret_cast<uintptr_t>(scratch) & 15) == 0;
        if (s.pool && !to_slices && scratch_floats < total) return hipErrorInvalidValue;
        float* sums = (s.pool || to_slices) ? scratch : out;
        a.out = sums;
        a.pool = 0;                                  // the slices write plain partial sums
        a.slice_stride = to_slices ? slice_stride : 0;
        if (to_slices) { a.bias = nullptr; a.relu = 0; }
        if (!to_slices && !(s.pre_zeroed == sums && s.pre_zeroed_count >= total))
            hipLaunchKernelGGL(fill_zero_kernel, dim3(fill_blocks), dim3(256), 0, stream, sums, total);
        // the finishing kernel below may clear the next launch's target on the way, unless that
        // is the very buffer it reads the sums from
        float* zero_next = (s.zero_next && s.zero_next != sums) ? s.zero_next : nullptr;
        const size_t zero_next_count = zero_next ? s.zero_next_count : 0;
        if (zero_next && s.zero_next_done) *s.zero_next_done = true;
        hipLaunchKernelGGL((tiled_conv_kernel<GEO, true>), dim3((unsigned)blocks, (unsigned)ksplit), dim3(64 * waves),
                           lds_bytes, stream, a);
        if (s.pool) {
            const int pho = s.ho / 2, pwo = s.wo / 2;
            const size_t ptotal = (size_t)s.n * s.c_out * pho * pwo;
            const unsigned pblocks = (unsigned)std::min<size_t>((std::max(ptotal, zero_next_count) + 255) / 256, 256 * 32);
            // max(relu(x + b)) over a window = relu(max(x) + b): one bias add and one ReLU per cell
            hipLaunchKernelGGL(bias_relu_pool_kernel, dim3(pblocks), dim3(256), 0, stream,
                               static_cast<const float*>(sums), bias, out, s.c_out, s.ho, s.wo, pho, pwo, ptotal,
                               make_fast_div((uint32_t)std::max(pwo, 1)), make_fast_div((uint32_t)std::max(pho, 1)),
                               make_fast_div((uint32_t)s.c_out), zero_next, zero_next_count,
                               to_slices ? ksplit : 1, slice_stride);
        } else {
            launch_bias_act(out, sums, to_slices ? ksplit : 1, slice_stride, bias, s.c_out, plane, total, s.relu,
                            zero_next, zero_next_count, stream);
        }
        return hipGetLastError();
    }
}

// X(name, G, PR, PC, S, TGX, DENSE, MAXSLOTS, MODE, EXPERIMENTAL) - one line per compiled variant
#include "variants.def"

#define X(name, G, PR, PC, S, TGX, DENSE, MAXSLOTS, MODE, EXPERIMENTAL)                    \
    using Geo_##name = Geo<G, PR, PC, S, TGX, DENSE, MAXSLOTS, MODE>;                      \
    using Stream_##name = std::conditional<DENSE, NoStream<G, PR, PC, S, TGX, MODE>,       \
                                           StreamLoop<G, PR, PC, S, TGX, ((MODE) & 15)>>::type;
PATDNN_VARIANTS
#undef X

static const TiledVariant kVariants[] = {
#define X(name, G, PR, PC, S, TGX, DENSE, MAXSLOTS, MODE, EXPERIMENTAL)                    \
    {#name, G, PR, PC, S, TGX, DENSE, ((MODE) & 1) != 0, ((MODE) & 2) != 0, EXPERIMENTAL != 0, MODE, ((MODE) & 16) ? 1 : 2, \
     Geo_##name::TILEP, Geo_##name::TILEP,                                                 \
     MAXSLOTS, Stream_##name::kBlockBytes, Stream_##name::kTableOff, Stream_##name::kCtrlBytes, \
     Stream_##name::kRecords, &launch_tiled<Geo_##name>},
    PATDNN_VARIANTS
#undef X
};

size_t split_slice_stride(size_t total) { return (total + 63) / 64 * 64; }

hipError_t launch_fill_zero(float* p, size_t count, hipStream_t stream)
{
    if (count == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((count + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, p, count);
    return hipGetLastError();
}

int num_tiled_variants() { return (int)(sizeof(kVariants) / sizeof(kVariants[0])); }
const TiledVariant& tiled_variant(int i) { return kVariants[i]; }

}  // namespace patdnn
