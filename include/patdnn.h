/*
 * patdnn.h - C ABI of the MI355X (gfx950) pattern-sparse 3x3 convolution library.
 *
 * The library runs the inference hot path of PatDNN (ASPLOS'20): 3x3 CONV layers
 * (paper section 2.1) whose weights obey the two constraints of section 4.2 - every
 * surviving kernel keeps only the four positions of one pattern out of a small
 * pattern set (section 3.1, 4.1), and whole kernels are removed (connectivity
 * pruning).  `patdnn_encode` is the offline stage of section 5 (filter-kernel
 * reorder, compact weight storage); `patdnn_conv2d` is the generated layer code.
 *
 * Conventions
 *   - All functions are extern "C", never throw, and return a patdnn_status_t
 *     (PATDNN_OK == 0).  `patdnn_last_error()` returns a thread-local text for the
 *     last failure on the calling thread.
 *   - HOST pointers are ordinary process memory; DEVICE pointers are HIP device
 *     memory on the device that was current when the handle was encoded.
 *   - Tensors are dense, contiguous, fp32.  Weights are OIHW, activations NCHW.
 *   - The operation is cross-correlation (no kernel flip), zero padding:
 *       out[n][co][oh][ow] = act(bias[co] + sum_{ci,kh,kw} Wm[co][ci][kh][kw]
 *                                 * in[n][ci][oh*stride+kh-pad][ow*stride+kw-pad])
 *     where Wm is W with every position outside the kernel's pattern, and every
 *     removed kernel, set to zero.  H_out = floor((H + 2*pad - 3)/stride) + 1.
 *   - Pattern masks: bit (3*kh + kw) set = position kept.  The four stored weights
 *     of a kernel are in ascending bit order.
 */
#ifndef PATDNN_H
#define PATDNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct patdnn_layer* patdnn_handle_t;

typedef enum {
    PATDNN_OK = 0,
    PATDNN_EINVAL = 1,        /* null pointer, non-positive size, bad stride/pad/groups */
    PATDNN_EPATTERN = 2,      /* pattern id out of range, mask popcount != 4, or (STRICT) a
                                 non-zero weight outside its pattern / in a removed kernel */
    PATDNN_ENOMEM = 3,        /* host allocation failed */
    PATDNN_EHIP = 4,          /* a HIP runtime call failed (no device, launch error, ...) */
    PATDNN_EUNSUPPORTED = 5   /* valid request that this build does not implement */
} patdnn_status_t;

/* patdnn_layer_desc_t.flags */
#define PATDNN_DENSE      0x1u  /* no pruning: ids and kernel_mask ignored, all nine taps kept
                                   (the paper leaves the first layer alone, section 4.2) */
#define PATDNN_STRICT     0x2u  /* reject weights that are non-zero where the constraints of
                                   section 4.2 require zero, instead of ignoring them */
#define PATDNN_HOST_ONLY  0x4u  /* build the layout in host memory only (no device needed);
                                   decode/stats/export work, conv2d/tune return PATDNN_EHIP */

typedef struct {
    int32_t c_out;                 /* number of filters */
    int32_t c_in;                  /* input channels */
    int32_t groups;                /* 1, or c_in (== c_out): depthwise, one kernel per filter */
    int32_t stride;                /* 1 or 2 */
    int32_t pad;                   /* 0 or 1 */
    int32_t num_patterns;          /* 1..255 (ignored with PATDNN_DENSE) */
    const uint16_t* pattern_masks; /* HOST [num_patterns]; each must have exactly 4 bits set
                                      below bit 9 and keep the centre (bit 4), section 4.1 */
    uint32_t flags;
} patdnn_layer_desc_t;

/*
 * Offline stage (paper section 5.2 filter-kernel reorder, 5.3 compact storage).
 * Reads the three host arrays, builds the reordered compressed layout and uploads
 * it; the caller may free its arrays as soon as the call returns.
 *   dense_weights  HOST [c_out][c_in/groups][3][3]
 *   pattern_ids    HOST [c_out][c_in/groups], each < num_patterns; not read where the
 *                  kernel is removed; NULL allowed with PATDNN_DENSE
 *   kernel_mask    HOST [c_out][c_in/groups], non-zero = kept; NULL = all kept
 *   out            receives the handle; set to NULL on failure
 * Weights outside a kernel's pattern and weights of removed kernels are ignored
 * (or rejected with PATDNN_STRICT).  A filter with no kept kernel is legal.
 */
patdnn_status_t patdnn_encode(const patdnn_layer_desc_t* desc, const float* dense_weights,
                              const uint8_t* pattern_ids, const uint8_t* kernel_mask,
                              patdnn_handle_t* out);

/*
 * The projection operators of the pattern-based pruning stage (section 4.1, 4.2), as host
 * utilities that turn any dense weight tensor into the arrays patdnn_encode takes.  All
 * pointers HOST; weights [c_out][kernels_per_filter][3][3] fp32.  Magnitudes and norms are
 * compared in double computed from the fp32 values, summed over positions 0..8 in order.
 *   patdnn_mine_patterns       the natural pattern of a kernel is its centre plus the three
 *       other positions of largest magnitude (equal magnitudes: lower position); the k most
 *       frequent natural patterns over all kernels, most frequent first (equal counts: lower
 *       mask), are written to pattern_masks [k]; *found = how many there are (<= k).
 *   patdnn_project_patterns    per kernel, the pattern of the set that retains the largest
 *       sum of squares (equal: lower id) - the Euclidean projection onto the pattern
 *       constraint; writes pattern_ids [c_out][kernels_per_filter] and, if `projected` is not
 *       NULL, the projected weights (positions outside the chosen pattern zeroed).
 *   patdnn_project_connectivity  kernel_mask = 1 for the min(alpha, all) kernels of largest
 *       L2 norm (equal norms: lower index co*kernels_per_filter + ci), 0 for the others - the
 *       Euclidean projection onto the connectivity constraint.
 */
patdnn_status_t patdnn_mine_patterns(const float* dense_weights, int32_t c_out, int32_t kernels_per_filter,
                                     int32_t k, uint16_t* pattern_masks, int32_t* found);
patdnn_status_t patdnn_project_patterns(const float* dense_weights, int32_t c_out, int32_t kernels_per_filter,
                                        const uint16_t* pattern_masks, int32_t num_patterns,
                                        uint8_t* pattern_ids, float* projected);
patdnn_status_t patdnn_project_connectivity(const float* dense_weights, int32_t c_out, int32_t kernels_per_filter,
                                            int64_t alpha, uint8_t* kernel_mask);

/*
 * The layer itself (section 2.1 CONV + ReLU; executed from the reordered layout as
 * in section 5.2-5.4).  Asynchronous on `stream`; allocates nothing, never
 * synchronises.
 *   input   DEVICE [n][c_in][h_in][w_in]
 *   bias    DEVICE [c_out], or NULL for no bias
 *   output  DEVICE [n][c_out][h_out][w_out]; must not overlap input
 *   stream  a hipStream_t (NULL = the default stream)
 * n == 0 is a no-op.  Tensors are limited to 2^31-1 elements per image
 * (c*h*w) and the whole call to what 64-bit offsets address.
 */
patdnn_status_t patdnn_conv2d(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                              int32_t w_in, const float* bias, float* output,
                              int32_t fuse_relu, void* stream);

/*
 * The layer on half-precision storage, as the paper's GPU runs keep weights and intermediate
 * results (section 6.1): `input` and `output` are DEVICE tensors of IEEE binary16 values
 * (same shapes and layout as patdnn_conv2d, 2 bytes per element), the weights are the
 * handle's fp32 weights rounded to binary16 (nearest, ties to even; done once by
 * patdnn_encode), the bias stays fp32, every product and sum is fp32, and the result is
 * rounded to binary16 once when it is stored.  Depthwise layers run the depthwise kernel
 * (bound by HBM bandwidth: half the bytes, about half the time); all other layers run the
 * filter-major FKW kernel - the tiled kernels are fp32 only.  Otherwise as patdnn_conv2d.
 */
patdnn_status_t patdnn_conv2d_f16(patdnn_handle_t h, const void* input, int32_t n, int32_t h_in, int32_t w_in,
                                  const float* bias, void* output, int32_t fuse_relu, void* stream);

/*
 * The layer followed by ReLU and 2x2 max pooling with stride 2 (an odd last row / column
 * is dropped), fused: the CONV stages of the networks the paper runs end in a pooling
 * layer (section 2.1, section 6.2) and only the pooled tensor is written.
 *   output  DEVICE [n][c_out][h_out/2][w_out/2]; must not overlap input
 * Two launches on `stream` (a kernel that zeroes the output, then the layer, whose lanes
 * fold their values into the pooled cells with integer atomic max on the float bits:
 * exact and independent of the order).  Otherwise as patdnn_conv2d.  Depthwise layers:
 * PATDNN_EUNSUPPORTED.  A layer whose configuration splits the input channels runs its
 * default configuration here.
 */
patdnn_status_t patdnn_conv2d_pool(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                                   int32_t w_in, const float* bias, float* output, void* stream);

/*
 * patdnn_conv2d / patdnn_conv2d_pool with a workspace from the caller, for layers whose
 * configuration splits the input channels into slices (`ksplit` > 1 of patdnn_config_t: the
 * way a layer with few output tiles fills the chip; section 5.5 leaves such launch
 * parameters to the tuner).  Without a workspace the slices add their partial sums into the
 * zeroed output with atomics (three launches: zero fill, the layer, bias + activation; the order
 * of the additions, and with it the last bits of the result, varies from run to run).  With
 * a workspace of patdnn_workspace_floats() floats every slice stores its partial sums to a
 * buffer of its own and the finishing kernel adds the buffers in slice order: two launches, no
 * atomics, and results that repeat bit for bit.
 *   pool2             non-zero: ReLU + 2x2 max pooling fused as in patdnn_conv2d_pool (`fuse_relu`
 *                     is then implied and `output` is the pooled tensor); a pooled layer
 *                     keeps its split configuration only with a workspace
 *   workspace         DEVICE, 16-byte aligned and apart from input and output (else
 *                     PATDNN_EINVAL), caller-owned, contents undefined before and after; may
 *                     be NULL (then as the plain calls)
 *   workspace_floats  its size; if it is smaller than the layer needs the call runs as
 *                     without one
 * Calls that share a workspace must not overlap in time.  Nothing is allocated.
 * patdnn_workspace_floats: what the handle's present configuration can use at this input
 * size (0: it does not split; also 0 for arguments that patdnn_conv2d would reject).
 */
size_t patdnn_workspace_floats(patdnn_handle_t h, int32_t n, int32_t h_in, int32_t w_in);
patdnn_status_t patdnn_conv2d_ws(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in, int32_t w_in,
                                 const float* bias, float* output, int32_t fuse_relu, int32_t pool2,
                                 float* workspace, size_t workspace_floats, void* stream);

/* out_nchw = {n, c_out, h_out, w_out}; PATDNN_EINVAL if the output would be empty. */
patdnn_status_t patdnn_output_shape(patdnn_handle_t h, int32_t n, int32_t h_in, int32_t w_in,
                                    int32_t out_nchw[4]);

/*
 * Inverse of encode, read back from the stored (device-resident) layout: the exact
 * fp32 bits at pattern positions of kept kernels and +0.0 elsewhere, the caller's
 * pattern id for every kept kernel (0 for removed ones and for dense layers), and
 * the 0/1 kernel mask.  Any output pointer may be NULL.  All HOST.
 */
patdnn_status_t patdnn_decode(patdnn_handle_t h, float* dense_weights, uint8_t* pattern_ids,
                              uint8_t* kernel_mask);

/*
 * The five arrays of the paper's FKW format (section 5.3) as stored for this
 * layer, copied to HOST buffers (any may be NULL to skip):
 *   offset  [c_out+1]  cumulative kept kernels per stored filter
 *   reorder [c_out]    original output channel of each stored filter
 *   index   [kept]     input channel of each stored kernel
 *   stride  [c_out][num_patterns+1]  cumulative kernels per pattern, per filter
 *   weight  [kept][taps]  taps = 4 (9 for a dense layer)
 * Sizes come from patdnn_layout_stats.
 */
patdnn_status_t patdnn_export_fkw(patdnn_handle_t h, int32_t* offset, int32_t* reorder,
                                  int32_t* index, int32_t* stride, float* weight);

/*
 * The layer as the conventional compressed-sparse-row matrix A[c_out][c_in*9] that the paper
 * compares its storage with (section 5.3, section 6.3) and that the "csr" kernel reads:
 * column = ci*9 + 3*kh + kw, the kept positions of every surviving kernel, ascending per
 * filter, filters in their original order.  `*nnz` receives the number of stored weights
 * (4 x kept kernels); row_ptr [c_out+1], col [nnz], val [nnz] are HOST buffers, any may be
 * NULL (call once with only `nnz` to size them).  Pruned, non-depthwise layers.
 */
patdnn_status_t patdnn_export_csr(patdnn_handle_t h, int64_t* nnz, int32_t* row_ptr, int32_t* col,
                                  float* val);

typedef struct {
    int64_t kept_kernels;      /* kernels that survived connectivity pruning */
    int32_t taps;              /* stored weights per kernel: 4, or 9 for a dense layer */
    int32_t num_patterns;      /* patterns of the layer (1 for dense) */
    int64_t fkw_weight_bytes;  /* weight array */
    int64_t fkw_index_bytes;   /* offset + reorder + index + stride arrays */
    int64_t tiled_bytes;       /* device bytes of the per-filter-group layouts the tiled kernels read */
    int32_t min_filter_length, max_filter_length;
    int32_t distinct_filter_lengths;
    int32_t filter_groups;     /* groups of the default tiled layout (0 if none) */
    int32_t group_size;        /* filters per group of that layout */
    int64_t max_group_kernels, min_group_kernels;   /* kept kernels in the fullest / emptiest group */
} patdnn_stats_t;

patdnn_status_t patdnn_layout_stats(patdnn_handle_t h, patdnn_stats_t* out);

/*
 * Launch configuration of one layer.  `variant` selects the kernel:
 *   0  PATDNN_VARIANT_FKW   filter-major walk of the FKW arrays, one lane per output
 *                           pixel (handles every shape; the reorder-only code of
 *                           section 5.2)
 *   >0 tiled variants       LDS-staged input tiles, register patches, filter groups
 *                           (section 5.4 load-redundancy elimination); see
 *                           patdnn_variant_name
 *   after the tiled ones    "dw_p1x4": depthwise layers (groups == c_in), one pass over
 *                           input and output with 16-byte accesses, four outputs per lane;
 *                           the default for such layers (section 6.1 evaluates MobileNet-V2)
 *                           "noopt", "csr": comparison kernels of the paper's evaluation, never
 *                           chosen by the library: the layer before filter-kernel reorder with
 *                           the pattern of every kernel decided inside the inner loop (the
 *                           "No-opt" stage of the per-layer breakdown, section 6.3), and the
 *                           layer as a CSR matrix (the control of section 6.2); pruned,
 *                           non-depthwise layers only
 * A configuration set with patdnn_set_config is taken as given or refused
 * (PATDNN_EUNSUPPORTED), never replaced by another one at launch time.
 * `ck` = input channels staged per LDS pass, `waves` = wavefronts (filter groups)
 * per workgroup; 0 lets the library choose.  `ksplit` > 1 (tiled sparse variants)
 * cuts the input channels into that many
 * slices handled by different workgroups, whose partial sums are added into the output
 * with atomic adds between a zero-fill and a bias + ReLU kernel (three launches; the
 * summation order then varies from run to run within fp32 rounding); 0 or 1 = off.
 * The environment variable PATDNN_WAVE_PRIORITY=0 (read once per process) switches off
 * the issue priorities that the tiled kernels give the workgroups of their last round; it
 * changes timing only, never results.
 */
typedef struct {
    int32_t variant;
    int32_t ck;
    int32_t waves;
    int32_t ksplit;
} patdnn_config_t;

#define PATDNN_VARIANT_FKW 0

int32_t         patdnn_num_variants(void);
const char*     patdnn_variant_name(int32_t variant);   /* NULL if out of range */
/* PATDNN_EUNSUPPORTED if the variant cannot run this layer (stride, depthwise, ...). */
patdnn_status_t patdnn_set_config(patdnn_handle_t h, const patdnn_config_t* cfg);
patdnn_status_t patdnn_get_config(patdnn_handle_t h, patdnn_config_t* cfg);

/*
 * Parameter auto-tuning (section 5.5), reduced to an exhaustive timed search over
 * the variants and launch parameters that can run this layer at this input size.
 * Runs every candidate on the caller's buffers (a few runs each; the fastest four again in
 * alternating turns, judged by the median of their turns; output ends up holding a valid
 * result of the winner), synchronises the stream, keeps the fastest in the handle and
 * reports its time.  `best_us` may be NULL.
 */
patdnn_status_t patdnn_tune(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                            int32_t w_in, const float* bias, float* output, void* stream,
                            float* best_us);
/*
 * The same search for callers of patdnn_conv2d_ws: candidates that split the input channels
 * are timed with the workspace (DEVICE, 16-byte aligned, caller-owned; those it is too small
 * for are timed as without one), so the configuration kept is the fastest for calls that
 * pass a workspace of this size.  NULL / 0: exactly patdnn_tune.
 */
patdnn_status_t patdnn_tune_ws(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                               int32_t w_in, const float* bias, float* output, float* workspace,
                               size_t workspace_floats, void* stream, float* best_us);

/*
 * The filter-group layout that a tiled sparse variant executes (section 5.2-5.4 as
 * laid out for this GPU), for inspection and round-trip tests.  `ck` as in
 * patdnn_config_t (0 = the variant's default).  The layout is built if the handle
 * does not hold it yet.
 *   A group is `G` filters that one wavefront computes; `slot_channel` gives the
 *   original output channel of each (group, slot), -1 for an unused slot.  Filters are
 *   assigned so that the groups carry equal work in every chunk (section 5.2: equal work
 *   for the units that wait for each other).
 *   Per group and per chunk of `ck` input channels, the low 28 bits of `chunk_ptr`
 *   give the first step; a step is 24 dwords and all its kernels read ONE input
 *   channel.  A kernel's code offset is
 *     table_off + ((set*G + slot)*56 + pattern index)*block_bytes,
 *   pattern index = rank of the pattern among the 56 centre-keeping four-entry
 *   patterns (section 4.1) ordered by their other three positions; set = window
 *   register set (0, or 0/1 with double_window).
 *   threaded == 0:
 *     0..15   four weights each of up to `records` (4) kernels
 *     16..19  per kernel its code offset; the entry after the last kernel holds
 *             3*ctrl_bytes or 4*ctrl_bytes ("step done", even / odd step of the chunk)
 *     20      what runs when the step starts, k*ctrl_bytes: k = 0 / 1 load a channel's
 *             window into set 0 / 1, 2 nothing, 5 end of the chunk's stream
 *     21      byte offset of that channel inside the staged chunk
 *             (channel index in the chunk * lds_channel_bytes)
 *   threaded == 1:
 *     6i..6i+5  record i < `records` (3): four weights, code offset, zero.  The record
 *             after the last kernel holds only an offset (after three kernels: dword 22):
 *             k*ctrl_bytes, the block that enters the NEXT step, k = 3*(step parity) +
 *             action (0 nothing, 1 / 2 load a window into set 0 / 1), or k = 6, the end
 *     23      byte offset, inside the staged chunk, of the channel the step's own entry
 *             block loads
 *     bits 28..31 of chunk_ptr: k of the block that enters the chunk's first step
 *   With double_window the window loaded when a step starts is the one the NEXT
 *   channel's kernels use, and a chunk's stream opens with a step that only loads.
 * patdnn_export_tiled copies the arrays to HOST buffers (read back from the device
 * unless the handle is host-only); any pointer may be NULL.
 */
typedef struct {
    int32_t G, num_groups, ck, num_chunks;
    int64_t num_steps;             /* steps array holds num_steps*24 dwords */
    uint32_t block_bytes, table_off, ctrl_bytes, records;
    int32_t double_window;
    int32_t lds_channel_bytes;
    int32_t threaded;
    int32_t patch_rows, patch_cols;   /* output patch of one lane */
    int32_t conv_stride;
    int32_t lanes_x;               /* lanes across a band; a wavefront covers 64/lanes_x bands */
    int32_t experimental;          /* needs PATDNN_EXPERIMENTAL=1 to run */
    int32_t mode;                  /* interpreter build: bit 0 double_window, bit 1 threaded,
                                      bit 2 window in fixed registers read two floats at a time */
} patdnn_tiled_info_t;

patdnn_status_t patdnn_tiled_info(patdnn_handle_t h, int32_t variant, int32_t ck,
                                  patdnn_tiled_info_t* out);
patdnn_status_t patdnn_export_tiled(patdnn_handle_t h, int32_t variant, int32_t ck,
                                    int32_t* slot_channel,   /* [num_groups*G] */
                                    uint32_t* chunk_ptr,     /* [num_groups*num_chunks] */
                                    uint32_t* steps);        /* [num_steps*24] */

/*
 * Device self-test behind the variants with threaded dispatch: checks on the current
 * device that scalar relative moves (the instruction those variants use to fetch the
 * next record, whose result becomes a jump address) behave as the generated code
 * assumes.  Runs one tiny kernel the first time (allocates and frees 20 bytes,
 * synchronises); later calls return the remembered result.  PATDNN_OK, or
 * PATDNN_EUNSUPPORTED with the reason in patdnn_last_error(); the library refuses to
 * build threaded layouts on a device that fails it.
 */
patdnn_status_t patdnn_selftest(void);

void        patdnn_destroy(patdnn_handle_t h);          /* NULL is a no-op */

/*
 * A stack of layers run back to back on one stream - the paper's headline scenario, one
 * image through all CONV layers of a network (section 6.2).  Layer i reads what layer
 * i-1 wrote; `pool2` fuses ReLU + 2x2 max pooling into the layer (as patdnn_conv2d_pool).
 * The stack owns two DEVICE buffers for the tensors between layers and one for partial sums
 * (allocated by patdnn_stack_create, freed by patdnn_stack_destroy): layers that are
 * configured, when the stack is created, to split their input channels get the workspace of
 * patdnn_conv2d_ws from it (one buffer per channel slice, up to 512 MB; a layer that would
 * need more, or is reconfigured later to need more than there is, adds its slices up with
 * atomics as patdnn_conv2d does).  Handles and bias arrays stay the caller's and must outlive
 * the stack.
 *   patdnn_stack_run, use_graph == 0: every launch goes to `stream` directly.
 *   use_graph != 0: the launches are recorded once into a HIP graph (stream capture on
 *   `stream`, which must not be the default stream; preceded by one plain run the first
 *   time) and replayed with a single graph launch on every later call with the same
 *   input / output addresses; other addresses record again.  No memset node is recorded:
 *   buffers are cleared by kernels.
 * Asynchronous; calls on one stack must not overlap.
 */
typedef struct patdnn_stack* patdnn_stack_t;
typedef struct {
    patdnn_handle_t layer;
    const float* bias;       /* DEVICE [c_out] or NULL */
    int32_t fuse_relu;
    int32_t pool2;           /* ReLU + 2x2 max pooling after the layer (implies fuse_relu) */
} patdnn_stack_layer_t;

patdnn_status_t patdnn_stack_create(const patdnn_stack_layer_t* layers, int32_t num_layers, int32_t n,
                                    int32_t h_in, int32_t w_in, patdnn_stack_t* out);
patdnn_status_t patdnn_stack_output_shape(patdnn_stack_t s, int32_t out_nchw[4]);
patdnn_status_t patdnn_stack_run(patdnn_stack_t s, const float* input, float* output,   /* DEVICE */
                                 int32_t use_graph, void* stream);
void            patdnn_stack_destroy(patdnn_stack_t s);     /* NULL is a no-op */

/*
 * patdnn_stack_run (use_graph == 0) for callers that must not allocate or cannot let a
 * library allocate on their behalf - code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: the tensors between the layers and the partial sums of
 * split layers live in a device array built into the library (32 MiB per GPU, held until the
 * process ends) instead of the stack's own buffers.  The call allocates and frees nothing.
 * PATDNN_EUNSUPPORTED (with the two sizes in patdnn_last_error) if the stack needs more
 * than the array holds: the sum, each rounded up to 256 bytes, of the largest tensor
 * written by the even-numbered layers, the largest written by the odd-numbered layers (the
 * last layer writes `output`) and the largest un-pooled output of a pooled layer.  If the
 * array also has room for one partial-sum buffer per channel slice (the stack's own third
 * buffer) the split layers use it as in patdnn_stack_run; otherwise they add their slices
 * up with atomics.  All calls on one GPU share the array: calls that overlap in time on the
 * same GPU race.  Results are those of patdnn_stack_run within the tolerance of a sum
 * taken in another order.
 */
patdnn_status_t patdnn_stack_run_static(patdnn_stack_t s, const float* input, float* output,   /* DEVICE */
                                        void* stream);
const char* patdnn_status_string(patdnn_status_t s);
const char* patdnn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PATDNN_H */
