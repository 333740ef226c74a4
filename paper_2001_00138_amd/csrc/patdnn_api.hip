// C ABI of the library (see include/patdnn.h): handle management, upload of the
// encoded layouts, variant selection, launch, decode, tuning.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <iterator>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "kernels.hpp"
#include "layout.hpp"

using namespace patdnn;

namespace {

thread_local std::string g_err;

patdnn_status_t fail(patdnn_status_t s, const std::string& msg)
{
    g_err = msg;
    return s;
}

patdnn_status_t hip_fail(hipError_t e, const char* what)
{
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return PATDNN_EHIP;
}

}  // namespace

namespace patdnn {
void set_last_error(const std::string& msg) { g_err = msg; }     // for the other translation units
}

namespace {

struct TiledOnDevice {
    Tiled host;
    DevTiled dev;
    std::vector<void*> allocations;       // device arrays of this layout
    ~TiledOnDevice()
    {
        for (void* p : allocations) (void)hipFree(p);
    }
};

}  // namespace

struct patdnn_layer {
    LayerHost L;
    bool on_device = false;
    int device = -1;
    DevFkw dfkw;
    // by (variant index, ck); dense variants use ck = 0
    std::map<std::pair<int, int>, std::unique_ptr<TiledOnDevice>> tiled;
    std::vector<void*> allocations;
    // the comparison kernels' layouts (built when such a variant is first selected)
    struct CompareHost {
        std::vector<int32_t> row_ptr, col, kmask;
        std::vector<float> val;
    } noopt_host, csr_host;
    DevCompare noopt_dev, csr_dev;
    bool compare_built = false, compare_on_device = false;
    patdnn_config_t cfg{-1, 0, 0, 1};                      // variant -1: choose per call
    bool cfg_tuned = false;                                // cfg came from patdnn_tune (for one input size)

    ~patdnn_layer()
    {
        for (void* p : allocations) (void)hipFree(p);
    }
};

namespace {

template <class T>
hipError_t upload(std::vector<void*>& owner, const std::vector<T>& v, const T** out, size_t extra = 0)
{
    *out = nullptr;
    const size_t bytes = (v.size() + extra) * sizeof(T);
    if (bytes == 0) return hipSuccess;
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) return e;
    owner.push_back(p);
    if (extra) {
        e = hipMemset(p, 0, bytes);
        if (e != hipSuccess) return e;
    }
    if (!v.empty()) {
        e = hipMemcpy(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
        if (e != hipSuccess) return e;
    }
    *out = static_cast<const T*>(p);
    return hipSuccess;
}

bool variant_fits_layer(const patdnn_layer* h, const TiledVariant& v)
{
    const LayerHost& L = h->L;
    if (L.depthwise) return false;
    if (v.dense != L.dense) return false;
    if (v.S != L.desc.stride) return false;
    if (!L.dense && !L.all_in_universe) return false;
    if (L.desc.c_in > 65535) return false;
    return true;
}

// Variants marked experimental have passed the host model of the interpreter but have not
// been measured on hardware; they run only when the caller asks for them by number AND the
// environment carries PATDNN_EXPERIMENTAL=1.
bool experimental_allowed()
{
    const char* e = std::getenv("PATDNN_EXPERIMENTAL");
    return e && e[0] == '1' && e[1] == 0;
}

bool variant_selectable(const patdnn_layer* h, const TiledVariant& v)
{
    return variant_fits_layer(h, v) && !v.experimental;
}

// Variant numbers: 0 the FKW walk, 1..T the tiled variants, then the kernels below.
enum ExtraVariant { kExtraDepthwise = 0, kExtraNoopt, kExtraCsr, kNumExtra };
int extra_variant(int variant) { return variant - 1 - num_tiled_variants(); }     // < 0: not one
int variant_of_extra(int extra) { return 1 + num_tiled_variants() + extra; }
const char* const kExtraNames[kNumExtra] = {"dw_p1x4", "noopt", "csr"};

constexpr int kMaxLdsBytes = 160 * 1024;      // LDS of one CU; two staging buffers must fit
constexpr int kMaxWaves = 8;

int default_ck(const TiledVariant& v, int c_in)
{
    const int max_ck = kMaxLdsBytes / (4 * v.lds_buffers * v.lds_floats_per_channel);
    return std::max(1, std::min(std::min(8, max_ck), c_in));
}

// Smallest / default launch parameters of a tiled variant for this layer; false if
// the variant cannot run at all.
bool resolve_tiled_params(const patdnn_layer* h, const TiledVariant& v, const ConvShape& s,
                          int32_t& ck, int32_t& waves)
{
    const int num_groups = (h->L.desc.c_out + v.G - 1) / v.G;
    const int min_waves = (v.stage_elems + 64 * v.max_slots - 1) / (64 * v.max_slots);
    if (min_waves > kMaxWaves) return false;
    if (waves <= 0) waves = std::max(min_waves, std::min(num_groups, 4));
    if (waves < min_waves || waves > kMaxWaves) return false;
    const int max_ck = kMaxLdsBytes / (4 * v.lds_buffers * v.lds_floats_per_channel);
    if (max_ck < 1) return false;
    if (ck <= 0) ck = default_ck(v, s.c_in);
    if (ck < 1 || ck > max_ck) return false;
    // staging offsets are 32-bit byte offsets relative to the first image of a tile
    const int nb = 64 / v.TGX;
    const long long span = (long long)(nb + 1) * s.c_in * s.h * s.w;
    if (span >= (1ll << 30)) return false;
    return true;
}

patdnn_status_t ensure_tiled(patdnn_layer* h, int vi, int ck, const DevTiled** out)
{
    const TiledVariant& v = tiled_variant(vi);
    if (v.dense) ck = 0;
    const std::pair<int, int> key(vi, ck);
    auto it = h->tiled.find(key);
    if (it == h->tiled.end()) {
        if (v.threaded && h->on_device) {
            std::string why;
            if (!movrel_selftest(why)) return fail(PATDNN_EUNSUPPORTED, "threaded variants are off: " + why);
        }
        std::unique_ptr<TiledOnDevice> t(new (std::nothrow) TiledOnDevice());
        if (!t) return fail(PATDNN_ENOMEM, "out of host memory");
        TiledParams prm;
        prm.G = v.G;
        prm.ck = ck;
        prm.block_bytes = v.block_bytes;
        prm.table_off = v.table_off;
        prm.ctrl_bytes = v.ctrl_bytes;
        prm.records = v.records;
        prm.double_window = v.double_window;
        prm.threaded = v.threaded;
        prm.channel_bytes = 4u * (uint32_t)v.lds_floats_per_channel;
        build_tiled(h->L, prm, t->host);
        if (t->host.overflow) return fail(PATDNN_EUNSUPPORTED, "layer has too many steps for this variant");
        t->dev.G = v.G;
        t->dev.num_groups = t->host.num_groups;
        t->dev.ck = ck;
        t->dev.num_chunks = t->host.num_chunks;
        if (h->on_device) {
            hipError_t e;
            if ((e = upload(t->allocations, t->host.slot_channel, &t->dev.slot_channel)) != hipSuccess ||
                (e = upload(t->allocations, t->host.chunk_ptr, &t->dev.chunk_ptr)) != hipSuccess ||
                (e = upload(t->allocations, t->host.steps, &t->dev.steps)) != hipSuccess ||
                (e = upload(t->allocations, t->host.w9, &t->dev.w9)) != hipSuccess)
                return hip_fail(e, "uploading the tiled layout");
        }
        it = h->tiled.emplace(key, std::move(t)).first;
    }
    if (out) *out = &it->second->dev;
    return PATDNN_OK;
}

// The layer before filter-kernel reorder (filters in original order, kernels by input
// channel, a pattern mask per kernel) and as a CSR matrix [c_out][c_in*9], both derived from
// the FKW arrays by undoing the reorder.
patdnn_status_t ensure_compare(patdnn_layer* h)
{
    if (h->L.depthwise || h->L.dense) return fail(PATDNN_EUNSUPPORTED, "the comparison kernels run pruned, non-depthwise layers");
    if (!h->compare_built) {
        const Fkw& f = h->L.fkw;
        const int c_out = h->L.desc.c_out, P = f.num_patterns;
        struct K { int32_t ci; int32_t mask; const float* w; };
        std::vector<std::vector<K>> per_filter((size_t)c_out);
        for (int s = 0; s < c_out; ++s) {
            const int32_t* st = &f.stride[(size_t)s * (P + 1)];
            for (int p = 0; p < P; ++p)
                for (int32_t k = f.offset[s] + st[p]; k < f.offset[s] + st[p + 1]; ++k)
                    per_filter[(size_t)f.reorder[s]].push_back(K{f.index[k], (int32_t)f.masks[p], &f.weight[(size_t)k * 4]});
        }
        auto& no = h->noopt_host;
        auto& cs = h->csr_host;
        no.row_ptr.assign(1, 0);
        cs.row_ptr.assign(1, 0);
        for (int co = 0; co < c_out; ++co) {
            auto& ks = per_filter[(size_t)co];
            std::sort(ks.begin(), ks.end(), [](const K& a, const K& b) { return a.ci < b.ci; });
            for (const K& k : ks) {
                no.col.push_back(k.ci);
                no.kmask.push_back(k.mask);
                int t = 0;
                for (int pos = 0; pos < 9; ++pos)
                    if ((k.mask >> pos) & 1) {
                        no.val.push_back(k.w[t]);
                        cs.col.push_back(k.ci * 9 + pos);
                        cs.val.push_back(k.w[t]);
                        ++t;
                    }
            }
            no.row_ptr.push_back((int32_t)no.col.size());
            cs.row_ptr.push_back((int32_t)cs.col.size());
        }
        h->compare_built = true;
    }
    if (h->on_device && !h->compare_on_device) {
        hipError_t e;
        if ((e = upload(h->allocations, h->noopt_host.row_ptr, &h->noopt_dev.row_ptr)) != hipSuccess ||
            (e = upload(h->allocations, h->noopt_host.col, &h->noopt_dev.col)) != hipSuccess ||
            (e = upload(h->allocations, h->noopt_host.kmask, &h->noopt_dev.kmask)) != hipSuccess ||
            (e = upload(h->allocations, h->noopt_host.val, &h->noopt_dev.val)) != hipSuccess ||
            (e = upload(h->allocations, h->csr_host.row_ptr, &h->csr_dev.row_ptr)) != hipSuccess ||
            (e = upload(h->allocations, h->csr_host.col, &h->csr_dev.col)) != hipSuccess ||
            (e = upload(h->allocations, h->csr_host.val, &h->csr_dev.val)) != hipSuccess)
            return hip_fail(e, "uploading the comparison layouts");
        h->compare_on_device = true;
    }
    return PATDNN_OK;
}

patdnn_status_t shape_of(const patdnn_layer* h, int32_t n, int32_t h_in, int32_t w_in, ConvShape& s)
{
    if (!h) return fail(PATDNN_EINVAL, "handle is NULL");
    if (n < 0 || h_in <= 0 || w_in <= 0) return fail(PATDNN_EINVAL, "n must be >= 0 and h_in, w_in positive");
    const auto& d = h->L.desc;
    s.n = n; s.c_in = d.c_in; s.c_out = d.c_out; s.h = h_in; s.w = w_in;
    s.stride = d.stride; s.pad = d.pad;
    s.ho = (h_in + 2 * d.pad - 3) / d.stride + 1;
    s.wo = (w_in + 2 * d.pad - 3) / d.stride + 1;
    s.relu = 0;
    if (h_in + 2 * d.pad < 3 || w_in + 2 * d.pad < 3 || s.ho <= 0 || s.wo <= 0)
        return fail(PATDNN_EINVAL, "input smaller than the 3x3 kernel");
    if ((long long)d.c_in * h_in * w_in > INT32_MAX || (long long)d.c_out * s.ho * s.wo > INT32_MAX)
        return fail(PATDNN_EUNSUPPORTED, "more than 2^31-1 elements per image");
    return PATDNN_OK;
}

// Launch with an explicit configuration (variant >= 0).
patdnn_status_t run_config(patdnn_layer* h, const patdnn_config_t& c, const ConvShape& s,
                           const float* in, const float* bias, float* out, hipStream_t stream,
                           float* scratch = nullptr, size_t scratch_floats = 0)
{
    if (c.variant == PATDNN_VARIANT_FKW) {
        hipError_t e = launch_fkw(h->dfkw, s, in, bias, out, stream);
        return e == hipSuccess ? PATDNN_OK : hip_fail(e, "launching the FKW kernel");
    }
    if (extra_variant(c.variant) == kExtraDepthwise) {
        if (!h->L.depthwise) return fail(PATDNN_EUNSUPPORTED, "the depthwise kernel runs depthwise layers only");
        hipError_t e = launch_dw(h->dfkw, s, in, bias, out, stream);
        return e == hipSuccess ? PATDNN_OK : hip_fail(e, "launching the depthwise kernel");
    }
    if (extra_variant(c.variant) == kExtraNoopt || extra_variant(c.variant) == kExtraCsr) {
        if (!h->compare_on_device) return fail(PATDNN_EUNSUPPORTED, "select the comparison kernel with patdnn_set_config first");
        if (s.pool) return fail(PATDNN_EUNSUPPORTED, "the comparison kernels have no pooled epilogue");
        const bool csr = extra_variant(c.variant) == kExtraCsr;
        hipError_t e = launch_compare(csr, csr ? h->csr_dev : h->noopt_dev, s, in, bias, out, stream);
        return e == hipSuccess ? PATDNN_OK : hip_fail(e, "launching a comparison kernel");
    }
    const int vi = c.variant - 1;
    if (vi < 0 || vi >= num_tiled_variants()) return fail(PATDNN_EINVAL, "no such variant");
    const TiledVariant& v = tiled_variant(vi);
    if (!variant_fits_layer(h, v)) return fail(PATDNN_EUNSUPPORTED, "variant cannot run this layer");
    if (v.experimental && !experimental_allowed())
        return fail(PATDNN_EUNSUPPORTED, "experimental variant: set PATDNN_EXPERIMENTAL=1 to run it");
    if (c.ksplit > 1 && v.dense) return fail(PATDNN_EUNSUPPORTED, "ksplit is for sparse variants");
    int32_t ck = c.ck, waves = c.waves;
    if (!resolve_tiled_params(h, v, s, ck, waves))
        return fail(PATDNN_EUNSUPPORTED, "launch parameters outside the variant's limits");
    const DevTiled* t = nullptr;
    // the layout of (variant, ck) is built by encode / set_config / tune, never here
    auto it = h->tiled.find(std::make_pair(vi, v.dense ? 0 : ck));
    if (it == h->tiled.end())
        return fail(PATDNN_EUNSUPPORTED, "no layout for this ck: choose it with patdnn_set_config");
    t = &it->second->dev;
    DevTiled dt = *t;
    if (v.dense) { dt.ck = ck; dt.num_chunks = (s.c_in + ck - 1) / ck; }
    if (c.ksplit > dt.num_chunks) return fail(PATDNN_EUNSUPPORTED, "ksplit exceeds the number of channel chunks");
    hipError_t e = v.launch(dt, s, in, bias, out, waves, c.ksplit, scratch, scratch_floats, stream);
    return e == hipSuccess ? PATDNN_OK : hip_fail(e, "launching a tiled kernel");
}

// Tiled variants in the order in which an untuned layer tries them: first the variant that the
// tuner prefers on most measured layers (threaded dispatch, 7x2 patch, one staging buffer; it
// needs the scalar relative moves that the self-test checks on the device), then the order
// of variants.def, whose first line (call dispatch) has no such requirement.
std::vector<int> default_variant_order(const patdnn_layer* h)
{
    std::vector<int> order;
    for (int vi = 0; vi < num_tiled_variants(); ++vi)
        if (std::string(tiled_variant(vi).name) == "t_g8_p7x2_s1_x8_thw1b") {
            std::string why;
            if (!h->on_device || movrel_selftest(why)) order.push_back(vi);
        }
    for (int vi = 0; vi < num_tiled_variants(); ++vi)
        if (order.empty() || vi != order[0]) order.push_back(vi);
    return order;
}

// The configuration used when the caller has not chosen or tuned one.
patdnn_config_t default_config(patdnn_layer* h, const ConvShape& s)
{
    if (h->L.depthwise) return patdnn_config_t{variant_of_extra(kExtraDepthwise), 0, 0, 1};
    for (int vi : default_variant_order(h)) {
        const TiledVariant& v = tiled_variant(vi);
        if (!variant_selectable(h, v)) continue;
        int32_t ck = 0, waves = 0;
        if (resolve_tiled_params(h, v, s, ck, waves)) return patdnn_config_t{vi + 1, ck, waves, 1};
    }
    return patdnn_config_t{PATDNN_VARIANT_FKW, 0, 0, 1};
}

}  // namespace

extern "C" {

patdnn_status_t patdnn_encode(const patdnn_layer_desc_t* desc, const float* dense_weights,
                              const uint8_t* pattern_ids, const uint8_t* kernel_mask,
                              patdnn_handle_t* out)
{
    if (out) *out = nullptr;
    if (!desc || !out) return fail(PATDNN_EINVAL, "desc / out is NULL");
    std::unique_ptr<patdnn_layer> h(new (std::nothrow) patdnn_layer());
    if (!h) return fail(PATDNN_ENOMEM, "out of host memory");
    std::string err;
    patdnn_status_t st;
    try {
        st = build_fkw(*desc, dense_weights, pattern_ids, kernel_mask, h->L, err);
    } catch (const std::bad_alloc&) {
        return fail(PATDNN_ENOMEM, "out of host memory");
    }
    if (st != PATDNN_OK) return fail(st, err);

    if (!(desc->flags & PATDNN_HOST_ONLY)) {
        hipError_t e = hipGetDevice(&h->device);
        if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
        const Fkw& f = h->L.fkw;
        if ((e = upload(h->allocations, f.offset, &h->dfkw.offset)) != hipSuccess ||
            (e = upload(h->allocations, f.reorder, &h->dfkw.reorder)) != hipSuccess ||
            (e = upload(h->allocations, f.index, &h->dfkw.index)) != hipSuccess ||
            (e = upload(h->allocations, f.stride, &h->dfkw.stride)) != hipSuccess ||
            (e = upload(h->allocations, f.weight, &h->dfkw.weight)) != hipSuccess ||
            (e = upload(h->allocations, f.masks, &h->dfkw.masks)) != hipSuccess)
            return hip_fail(e, "uploading the FKW arrays");
        h->dfkw.num_patterns = f.num_patterns;
        h->dfkw.taps = f.taps;
        {
            // the weights once more in binary16 (round to nearest even) for patdnn_conv2d_f16
            std::vector<uint16_t> w16(f.weight.size());
            for (size_t i = 0; i < w16.size(); ++i) {
                const _Float16 hv = static_cast<_Float16>(f.weight[i]);
                std::memcpy(&w16[i], &hv, 2);
            }
            const uint16_t* dev16 = nullptr;
            if ((e = upload(h->allocations, w16, &dev16)) != hipSuccess) return hip_fail(e, "uploading the binary16 weights");
            h->dfkw.weight_f16 = dev16;
        }
        if (h->L.depthwise) {
            // per stored filter: the mask of its kernel's pattern and its four weights
            const int c = desc->c_out, P = f.num_patterns;
            std::vector<int32_t> dmask((size_t)c, 0);
            std::vector<float> dweight((size_t)c * 4, 0.0f);
            for (int s = 0; s < c; ++s) {
                if (f.offset[s + 1] == f.offset[s]) continue;
                const int32_t* st = &f.stride[(size_t)s * (P + 1)];
                for (int p = 0; p < P; ++p)
                    if (st[p + 1] > st[p]) dmask[s] = f.masks[p];
                for (int t = 0; t < 4; ++t) dweight[(size_t)s * 4 + t] = f.weight[(size_t)f.offset[s] * 4 + t];
            }
            std::vector<uint16_t> dweight16(dweight.size());
            for (size_t i = 0; i < dweight16.size(); ++i) {
                const _Float16 hv = static_cast<_Float16>(dweight[i]);
                std::memcpy(&dweight16[i], &hv, 2);
            }
            const uint16_t* dev16 = nullptr;
            if ((e = upload(h->allocations, dmask, &h->dfkw.dw_mask)) != hipSuccess ||
                (e = upload(h->allocations, dweight, &h->dfkw.dw_weight)) != hipSuccess ||
                (e = upload(h->allocations, dweight16, &dev16)) != hipSuccess)
                return hip_fail(e, "uploading the depthwise arrays");
            h->dfkw.dw_weight_f16 = dev16;
        }
        h->on_device = true;
    }
    // build (and upload) the group layout of the default variant; the layouts of the other
    // variants are built when patdnn_set_config or patdnn_tune asks for them
    try {
        for (int vi : default_variant_order(h.get()))
            if (variant_selectable(h.get(), tiled_variant(vi))) {
                st = ensure_tiled(h.get(), vi, default_ck(tiled_variant(vi), desc->c_in), nullptr);
                if (st != PATDNN_OK) return st;
                break;
            }
    } catch (const std::bad_alloc&) {
        return fail(PATDNN_ENOMEM, "out of host memory");
    }
    *out = h.release();
    return PATDNN_OK;
}

patdnn_status_t patdnn_output_shape(patdnn_handle_t h, int32_t n, int32_t h_in, int32_t w_in,
                                    int32_t out_nchw[4])
{
    ConvShape s{};
    patdnn_status_t st = shape_of(h, n, h_in, w_in, s);
    if (st != PATDNN_OK) return st;
    if (!out_nchw) return fail(PATDNN_EINVAL, "out_nchw is NULL");
    out_nchw[0] = n; out_nchw[1] = s.c_out; out_nchw[2] = s.ho; out_nchw[3] = s.wo;
    return PATDNN_OK;
}

// What one layer of a stack hands to the next about zero fills: the region the next layer must
// find zeroed, which this layer clears in its finishing kernel if it has one (`done` tells).
struct ZeroRegion {
    float* p = nullptr;
    size_t count = 0;
};
struct ZeroHandoff {
    ZeroRegion pre_zeroed;   // in: already holds zeros when the layer starts
    ZeroRegion next;         // in: what the next layer will want zeroed
    bool done = false;       // out: `next` was cleared by this layer
};

// A split launch stores its slices to buffers of their own (no zero fill, no atomics) if the
// scratch holds one per slice; the launcher decides by the same rule.
static bool slices_fit(const float* scratch, size_t scratch_floats, int32_t ksplit, size_t full)
{
    return scratch && ksplit > 1 && (reinterpret_cast<uintptr_t>(scratch) & 15) == 0 &&
           scratch_floats / (size_t)ksplit >= split_slice_stride(full);
}

// The region that conv2d_impl must clear before this layer's kernels run (none: p == NULL).
// Mirrors the decisions of conv2d_impl below.
static ZeroRegion zero_need(patdnn_handle_t h, int32_t n, int32_t h_in, int32_t w_in, int32_t pool, float* output,
                            float* scratch, size_t scratch_floats)
{
    ConvShape s{};
    if (shape_of(h, n, h_in, w_in, s) != PATDNN_OK || !h->on_device || n == 0) return ZeroRegion{};
    const patdnn_config_t& c = h->cfg;
    const bool split = c.variant > 0 && c.ksplit > 1;
    const size_t full = (size_t)n * s.c_out * s.ho * s.wo;
    if (split && slices_fit(scratch, scratch_floats, c.ksplit, full)) return ZeroRegion{};   // stores only
    if (!pool) return split ? ZeroRegion{output, full} : ZeroRegion{};
    if (split && scratch && scratch_floats >= full) return ZeroRegion{scratch, full};
    return ZeroRegion{output, (size_t)n * s.c_out * (s.ho / 2) * (s.wo / 2)};
}

// `scratch` (DEVICE, `scratch_floats` floats, may be NULL): where a layer whose configuration
// splits the input channels keeps its partial sums: one buffer per slice if there is room
// (ksplit * split_slice_stride([n][c_out][ho][wo]) floats), else - pooled layers only - one
// buffer that the slices add into ([n][c_out][ho][wo]).
static patdnn_status_t conv2d_impl(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                                   int32_t w_in, const float* bias, float* output, int32_t fuse_relu,
                                   int32_t pool, hipStream_t stream, float* scratch = nullptr,
                                   size_t scratch_floats = 0, ZeroHandoff* handoff = nullptr)
{
    ConvShape s{};
    patdnn_status_t st = shape_of(h, n, h_in, w_in, s);
    if (st != PATDNN_OK) return st;
    if (!h->on_device) return fail(PATDNN_EHIP, "handle was encoded with PATDNN_HOST_ONLY");
    const int oh = pool ? s.ho / 2 : s.ho, ow = pool ? s.wo / 2 : s.wo;
    if (pool && (oh == 0 || ow == 0)) return fail(PATDNN_EINVAL, "output smaller than one 2x2 pooling window");
    if (pool && h->L.depthwise) return fail(PATDNN_EUNSUPPORTED, "fused pooling is not built for depthwise layers");
    if (n == 0) return PATDNN_OK;
    if (!input || !output) return fail(PATDNN_EINVAL, "input / output is NULL");
    {
        const char* in_lo = reinterpret_cast<const char*>(input);
        const char* in_hi = in_lo + 4ull * (size_t)n * s.c_in * s.h * s.w;
        const char* out_lo = reinterpret_cast<const char*>(output);
        const char* out_hi = out_lo + 4ull * (size_t)n * s.c_out * oh * ow;
        if (in_lo < out_hi && out_lo < in_hi) return fail(PATDNN_EINVAL, "output overlaps input");
    }
    s.relu = (fuse_relu || pool) ? 1 : 0;
    s.pool = pool ? 1 : 0;
    if (handoff) {
        s.pre_zeroed = handoff->pre_zeroed.p;
        s.pre_zeroed_count = handoff->pre_zeroed.count;
        s.zero_next = handoff->next.p;
        s.zero_next_count = handoff->next.count;
        s.zero_next_done = &handoff->done;
    }
    patdnn_config_t c = h->cfg;
    // a pooled layer that splits the input channels needs room for its partial sums; without
    // it the layer runs its default configuration
    const bool split_pool = pool && c.variant > 0 && c.ksplit > 1;
    const bool have_room = scratch && scratch_floats >= (size_t)n * s.c_out * s.ho * s.wo;
    if (c.variant < 0 || (split_pool && !have_room)) c = default_config(h, s);
    if (pool && !(split_pool && have_room) &&
        !(s.pre_zeroed == output && s.pre_zeroed_count >= (size_t)n * s.c_out * oh * ow)) {
        hipError_t e = launch_fill_zero(output, (size_t)n * s.c_out * oh * ow, stream);
        if (e != hipSuccess) return hip_fail(e, "zeroing the pooled output");
    }
    st = run_config(h, c, s, input, bias, output, stream, scratch, scratch_floats);
    if (st == PATDNN_EUNSUPPORTED && h->cfg.variant > 0 && h->cfg_tuned) {
        // a configuration tuned for another input size may not fit this one; a configuration
        // the caller set explicitly is never replaced: the error goes back instead
        c = default_config(h, s);
        if (pool && split_pool && have_room) {
            hipError_t e = launch_fill_zero(output, (size_t)n * s.c_out * oh * ow, stream);
            if (e != hipSuccess) return hip_fail(e, "zeroing the pooled output");
        }
        st = run_config(h, c, s, input, bias, output, stream, scratch, scratch_floats);
    }
    return st;
}

patdnn_status_t patdnn_conv2d(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                              int32_t w_in, const float* bias, float* output, int32_t fuse_relu,
                              void* stream)
{
    return conv2d_impl(h, input, n, h_in, w_in, bias, output, fuse_relu, 0, static_cast<hipStream_t>(stream));
}

size_t patdnn_workspace_floats(patdnn_handle_t h, int32_t n, int32_t h_in, int32_t w_in)
{
    ConvShape s{};
    if (shape_of(h, n, h_in, w_in, s) != PATDNN_OK) return 0;
    const patdnn_config_t& c = h->cfg;
    if (!(c.variant > 0 && c.ksplit > 1)) return 0;
    return (size_t)c.ksplit * split_slice_stride((size_t)n * s.c_out * s.ho * s.wo);
}

patdnn_status_t patdnn_conv2d_ws(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in, int32_t w_in,
                                 const float* bias, float* output, int32_t fuse_relu, int32_t pool2,
                                 float* workspace, size_t workspace_floats, void* stream)
{
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 15))
        return fail(PATDNN_EINVAL, "workspace must be 16-byte aligned");
    ConvShape s{};
    if (workspace && workspace_floats && input && output && shape_of(h, n, h_in, w_in, s) == PATDNN_OK) {
        const char* lo = reinterpret_cast<const char*>(workspace);
        const char* hi = lo + 4ull * workspace_floats;
        const char* in_lo = reinterpret_cast<const char*>(input);
        const char* in_hi = in_lo + 4ull * (size_t)n * s.c_in * s.h * s.w;
        const char* out_lo = reinterpret_cast<const char*>(output);
        const char* out_hi = out_lo + 4ull * (size_t)n * s.c_out * (pool2 ? s.ho / 2 : s.ho) * (pool2 ? s.wo / 2 : s.wo);
        if ((lo < in_hi && in_lo < hi) || (lo < out_hi && out_lo < hi))
            return fail(PATDNN_EINVAL, "workspace overlaps input or output");
    }
    return conv2d_impl(h, input, n, h_in, w_in, bias, output, pool2 ? 1 : fuse_relu, pool2 ? 1 : 0,
                       static_cast<hipStream_t>(stream), workspace, workspace ? workspace_floats : 0);
}

patdnn_status_t patdnn_conv2d_f16(patdnn_handle_t h, const void* input, int32_t n, int32_t h_in, int32_t w_in,
                                  const float* bias, void* output, int32_t fuse_relu, void* stream)
{
    ConvShape s{};
    patdnn_status_t st = shape_of(h, n, h_in, w_in, s);
    if (st != PATDNN_OK) return st;
    if (!h->on_device) return fail(PATDNN_EHIP, "handle was encoded with PATDNN_HOST_ONLY");
    if (n == 0) return PATDNN_OK;
    if (!input || !output) return fail(PATDNN_EINVAL, "input / output is NULL");
    if ((reinterpret_cast<uintptr_t>(input) | reinterpret_cast<uintptr_t>(output)) & 1u)
        return fail(PATDNN_EINVAL, "binary16 tensors must be 2-byte aligned");
    {
        const char* in_lo = static_cast<const char*>(input);
        const char* in_hi = in_lo + 2ull * (size_t)n * s.c_in * s.h * s.w;
        const char* out_lo = static_cast<const char*>(output);
        const char* out_hi = out_lo + 2ull * (size_t)n * s.c_out * s.ho * s.wo;
        if (in_lo < out_hi && out_lo < in_hi) return fail(PATDNN_EINVAL, "output overlaps input");
    }
    s.relu = fuse_relu ? 1 : 0;
    hipError_t e = h->L.depthwise
                       ? launch_dw_f16(h->dfkw, s, input, bias, output, static_cast<hipStream_t>(stream))
                       : launch_fkw_f16(h->dfkw, s, input, bias, output, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PATDNN_OK : hip_fail(e, "launching a binary16 kernel");
}

patdnn_status_t patdnn_conv2d_pool(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                                   int32_t w_in, const float* bias, float* output, void* stream)
{
    return conv2d_impl(h, input, n, h_in, w_in, bias, output, 1, 1, static_cast<hipStream_t>(stream));
}

patdnn_status_t patdnn_decode(patdnn_handle_t h, float* dense_weights, uint8_t* pattern_ids,
                              uint8_t* kernel_mask)
{
    if (!h) return fail(PATDNN_EINVAL, "handle is NULL");
    try {
        if (!h->on_device) {
            decode_fkw(h->L, h->L.fkw, dense_weights, pattern_ids, kernel_mask);
            return PATDNN_OK;
        }
        // read the five arrays back from device memory and invert them
        Fkw f;
        const Fkw& ref = h->L.fkw;
        f.taps = ref.taps;
        f.num_patterns = ref.num_patterns;
        f.offset.resize(ref.offset.size());
        f.reorder.resize(ref.reorder.size());
        f.index.resize(ref.index.size());
        f.stride.resize(ref.stride.size());
        f.weight.resize(ref.weight.size());
        f.masks.resize(ref.masks.size());
        auto back = [](void* dst, const void* src, size_t bytes) -> hipError_t {
            return bytes ? hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost) : hipSuccess;
        };
        hipError_t e;
        if ((e = back(f.offset.data(), h->dfkw.offset, f.offset.size() * 4)) != hipSuccess ||
            (e = back(f.reorder.data(), h->dfkw.reorder, f.reorder.size() * 4)) != hipSuccess ||
            (e = back(f.index.data(), h->dfkw.index, f.index.size() * 4)) != hipSuccess ||
            (e = back(f.stride.data(), h->dfkw.stride, f.stride.size() * 4)) != hipSuccess ||
            (e = back(f.weight.data(), h->dfkw.weight, f.weight.size() * 4)) != hipSuccess ||
            (e = back(f.masks.data(), h->dfkw.masks, f.masks.size() * 2)) != hipSuccess)
            return hip_fail(e, "reading the FKW arrays back");
        decode_fkw(h->L, f, dense_weights, pattern_ids, kernel_mask);
    } catch (const std::bad_alloc&) {
        return fail(PATDNN_ENOMEM, "out of host memory");
    }
    return PATDNN_OK;
}

patdnn_status_t patdnn_export_fkw(patdnn_handle_t h, int32_t* offset, int32_t* reorder,
                                  int32_t* index, int32_t* stride, float* weight)
{
    if (!h) return fail(PATDNN_EINVAL, "handle is NULL");
    const Fkw& f = h->L.fkw;
    auto get = [&](void* dst, const void* dev, const void* host, size_t bytes) -> hipError_t {
        if (!dst || !bytes) return hipSuccess;
        if (h->on_device) return hipMemcpy(dst, dev, bytes, hipMemcpyDeviceToHost);
        std::memcpy(dst, host, bytes);
        return hipSuccess;
    };
    hipError_t e;
    if ((e = get(offset, h->dfkw.offset, f.offset.data(), f.offset.size() * 4)) != hipSuccess ||
        (e = get(reorder, h->dfkw.reorder, f.reorder.data(), f.reorder.size() * 4)) != hipSuccess ||
        (e = get(index, h->dfkw.index, f.index.data(), f.index.size() * 4)) != hipSuccess ||
        (e = get(stride, h->dfkw.stride, f.stride.data(), f.stride.size() * 4)) != hipSuccess ||
        (e = get(weight, h->dfkw.weight, f.weight.data(), f.weight.size() * 4)) != hipSuccess)
        return hip_fail(e, "reading the FKW arrays back");
    return PATDNN_OK;
}

patdnn_status_t patdnn_export_csr(patdnn_handle_t h, int64_t* nnz, int32_t* row_ptr, int32_t* col, float* val)
{
    if (!h) return fail(PATDNN_EINVAL, "handle is NULL");
    try {
        patdnn_status_t st = ensure_compare(h);
        if (st != PATDNN_OK) return st;
    } catch (const std::bad_alloc&) {
        return fail(PATDNN_ENOMEM, "out of host memory");
    }
    const auto& c = h->csr_host;
    if (nnz) *nnz = (int64_t)c.col.size();
    auto get = [&](void* dst, const void* dev, const void* host, size_t bytes) -> hipError_t {
        if (!dst || !bytes) return hipSuccess;
        if (h->on_device) return hipMemcpy(dst, dev, bytes, hipMemcpyDeviceToHost);
        std::memcpy(dst, host, bytes);
        return hipSuccess;
    };
    hipError_t e;
    if ((e = get(row_ptr, h->csr_dev.row_ptr, c.row_ptr.data(), c.row_ptr.size() * 4)) != hipSuccess ||
        (e = get(col, h->csr_dev.col, c.col.data(), c.col.size() * 4)) != hipSuccess ||
        (e = get(val, h->csr_dev.val, c.val.data(), c.val.size() * 4)) != hipSuccess)
        return hip_fail(e, "reading the CSR arrays back");
    return PATDNN_OK;
}

patdnn_status_t patdnn_layout_stats(patdnn_handle_t h, patdnn_stats_t* out)
{
    if (!h || !out) return fail(PATDNN_EINVAL, "handle / out is NULL");
    const Fkw& f = h->L.fkw;
    std::memset(out, 0, sizeof(*out));
    out->kept_kernels = h->L.kept;
    out->taps = f.taps;
    out->num_patterns = f.num_patterns;
    out->fkw_weight_bytes = (int64_t)f.weight.size() * 4;
    out->fkw_index_bytes = 4 * (int64_t)(f.offset.size() + f.reorder.size() + f.index.size() + f.stride.size());
    std::vector<int32_t> len;
    for (size_t s = 0; s + 1 < f.offset.size(); ++s) len.push_back(f.offset[s + 1] - f.offset[s]);
    if (!len.empty()) {
        out->min_filter_length = *std::min_element(len.begin(), len.end());
        out->max_filter_length = *std::max_element(len.begin(), len.end());
        std::sort(len.begin(), len.end());
        out->distinct_filter_lengths = (int32_t)(std::unique(len.begin(), len.end()) - len.begin());
    }
    for (const auto& kv : h->tiled) out->tiled_bytes += (int64_t)kv.second->host.bytes();
    if (!h->tiled.empty()) {
        const Tiled& t = h->tiled.begin()->second->host;
        out->filter_groups = t.num_groups;
        out->group_size = t.G;
        if (!t.group_kernels.empty()) {
            out->max_group_kernels = *std::max_element(t.group_kernels.begin(), t.group_kernels.end());
            out->min_group_kernels = *std::min_element(t.group_kernels.begin(), t.group_kernels.end());
        }
    }
    return PATDNN_OK;
}

int32_t patdnn_num_variants(void) { return 1 + num_tiled_variants() + kNumExtra; }

const char* patdnn_variant_name(int32_t variant)
{
    if (variant == PATDNN_VARIANT_FKW) return "fkw";
    if (variant < 0 || variant >= patdnn_num_variants()) return nullptr;
    if (extra_variant(variant) >= 0) return kExtraNames[extra_variant(variant)];
    return tiled_variant(variant - 1).name;
}

patdnn_status_t patdnn_set_config(patdnn_handle_t h, const patdnn_config_t* cfg)
{
    if (!h || !cfg) return fail(PATDNN_EINVAL, "handle / cfg is NULL");
    if (cfg->variant < 0) {               // back to automatic choice
        h->cfg = patdnn_config_t{-1, 0, 0, 1};
        h->cfg_tuned = false;
        return PATDNN_OK;
    }
    if (cfg->variant >= patdnn_num_variants()) return fail(PATDNN_EINVAL, "no such variant");
    if (extra_variant(cfg->variant) == kExtraDepthwise) {
        if (!h->L.depthwise) return fail(PATDNN_EUNSUPPORTED, "the depthwise kernel runs depthwise layers only");
        h->cfg = patdnn_config_t{cfg->variant, 0, 0, 1};
        h->cfg_tuned = false;
        return PATDNN_OK;
    }
    if (extra_variant(cfg->variant) == kExtraNoopt || extra_variant(cfg->variant) == kExtraCsr) {
        try {
            patdnn_status_t st = ensure_compare(h);
            if (st != PATDNN_OK) return st;
        } catch (const std::bad_alloc&) {
            return fail(PATDNN_ENOMEM, "out of host memory");
        }
        h->cfg = patdnn_config_t{cfg->variant, 0, 0, 1};
        h->cfg_tuned = false;
        return PATDNN_OK;
    }
    if (cfg->variant > 0) {
        const TiledVariant& v = tiled_variant(cfg->variant - 1);
        if (!variant_fits_layer(h, v)) return fail(PATDNN_EUNSUPPORTED, "variant cannot run this layer");
        if (v.experimental && h->on_device && !experimental_allowed())
            return fail(PATDNN_EUNSUPPORTED, "experimental variant: set PATDNN_EXPERIMENTAL=1 to run it");
        if (cfg->ck < 0 || cfg->waves < 0 || cfg->waves > kMaxWaves || cfg->ksplit < 0 || cfg->ksplit > 64)
            return fail(PATDNN_EINVAL, "ck / waves / ksplit out of range");
        if (cfg->ksplit > 1 && v.dense) return fail(PATDNN_EUNSUPPORTED, "ksplit: sparse variants only");
        const int min_waves = (v.stage_elems + 64 * v.max_slots - 1) / (64 * v.max_slots);
        if (cfg->waves && cfg->waves < min_waves)
            return fail(PATDNN_EUNSUPPORTED, "too few wavefronts to stage a tile");
        if (cfg->ck && cfg->ck * 4 * v.lds_buffers * v.lds_floats_per_channel > kMaxLdsBytes)
            return fail(PATDNN_EUNSUPPORTED, "ck exceeds the LDS budget");
    }
    patdnn_config_t c = *cfg;
    if (c.ksplit < 1 || c.variant <= 0) c.ksplit = 1;
    if (c.variant > 0) {
        const TiledVariant& v = tiled_variant(c.variant - 1);
        if (c.ck == 0) c.ck = default_ck(v, h->L.desc.c_in);
        c.ck = std::min(c.ck, h->L.desc.c_in);
        try {
            patdnn_status_t st = ensure_tiled(h, c.variant - 1, c.ck, nullptr);
            if (st != PATDNN_OK) return st;
        } catch (const std::bad_alloc&) {
            return fail(PATDNN_ENOMEM, "out of host memory");
        }
        // an explicit configuration is taken as given or refused, never replaced at launch time
        const int num_chunks = v.dense ? (h->L.desc.c_in + c.ck - 1) / c.ck
                                       : h->tiled.find(std::make_pair(c.variant - 1, c.ck))->second->host.num_chunks;
        if (c.ksplit > num_chunks) return fail(PATDNN_EUNSUPPORTED, "ksplit exceeds the number of channel chunks");
    }
    h->cfg = c;
    h->cfg_tuned = false;
    return PATDNN_OK;
}

patdnn_status_t patdnn_get_config(patdnn_handle_t h, patdnn_config_t* cfg)
{
    if (!h || !cfg) return fail(PATDNN_EINVAL, "handle / cfg is NULL");
    *cfg = h->cfg;
    return PATDNN_OK;
}

patdnn_status_t patdnn_tune(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                            int32_t w_in, const float* bias, float* output, void* stream_,
                            float* best_us)
{
    return patdnn_tune_ws(h, input, n, h_in, w_in, bias, output, nullptr, 0, stream_, best_us);
}

patdnn_status_t patdnn_tune_ws(patdnn_handle_t h, const float* input, int32_t n, int32_t h_in,
                               int32_t w_in, const float* bias, float* output, float* workspace,
                               size_t workspace_floats, void* stream_, float* best_us)
{
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 15))
        return fail(PATDNN_EINVAL, "workspace must be 16-byte aligned");
    if (!workspace) workspace_floats = 0;
    ConvShape s{};
    patdnn_status_t st = shape_of(h, n, h_in, w_in, s);
    if (st != PATDNN_OK) return st;
    if (!h->on_device) return fail(PATDNN_EHIP, "handle was encoded with PATDNN_HOST_ONLY");
    if (n == 0 || !input || !output) return fail(PATDNN_EINVAL, "tuning needs n > 0 and real buffers");
    hipStream_t stream = static_cast<hipStream_t>(stream_);

    std::vector<patdnn_config_t> cands;
    // The grid: chunk sizes 8, 10 and 16 (smaller ones lose to their barrier count, larger ones
    // to LDS occupancy on every layer measured; 10 is the most that leaves the single-buffer 7x2
    // variant three workgroups per CU), 4 or 8 wavefronts per workgroup (fewer only when
    // the layer has fewer filter groups), and input-channel slices only for launches that
    // cannot fill the chip's wavefront slots three times over.
    const int ck_opts[] = {8, 10, 16};
    const int wave_opts[] = {1, 2, 4, 8};
    const long long kWaveSlots = 256 * 4 * 3;
    for (int vi = 0; vi < num_tiled_variants(); ++vi) {
        const TiledVariant& v = tiled_variant(vi);
        if (!(variant_selectable(h, v) || (experimental_allowed() && variant_fits_layer(h, v)))) continue;
        const int groups = (s.c_out + v.G - 1) / v.G;
        const long long bands = (long long)s.n * ((s.wo + v.TGX * v.PC - 1) / (v.TGX * v.PC)) * ((s.ho + v.PR - 1) / v.PR);
        const long long wavefronts = (bands + 64 / v.TGX - 1) / (64 / v.TGX) * groups;
        for (int ck : ck_opts)
            for (int waves : wave_opts) {
                int32_t ck2 = std::min(ck, s.c_in), w2 = waves;
                if (w2 < 4 && groups >= 4) continue;           // small workgroups only for few groups
                if (w2 > 1 && w2 / 2 >= groups) continue;      // mostly idle wavefronts
                if (!resolve_tiled_params(h, v, s, ck2, w2)) continue;
                const int num_chunks = (s.c_in + ck2 - 1) / ck2;
                for (int ks : {1, 2, 3, 4, 6, 8, 12, 16, 24, 32}) {
                    // slices only while the launch before this split leaves wavefront slots empty
                    if (ks > 1 && (v.dense || ks > num_chunks || wavefronts * (ks - 1) >= 2 * kWaveSlots)) continue;
                    patdnn_config_t c{vi + 1, ck2, w2, ks};
                    bool dup = false;
                    for (const auto& o : cands)
                        dup |= (o.variant == c.variant && o.ck == c.ck && o.waves == c.waves && o.ksplit == c.ksplit);
                    if (!dup && ensure_tiled(h, vi, ck2, nullptr) == PATDNN_OK) cands.push_back(c);
                }
            }
    }
    if (h->L.depthwise) cands.push_back(patdnn_config_t{variant_of_extra(kExtraDepthwise), 0, 0, 1});
    cands.push_back(patdnn_config_t{PATDNN_VARIANT_FKW, 0, 0, 1});

    hipEvent_t e0, e1;
    hipError_t e;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return hip_fail(e, "hipEventCreate");
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e, "hipEventCreate"); }
    float best = -1.0f;
    patdnn_config_t best_cfg = cands.back();
    patdnn_status_t result = PATDNN_OK;
    // milliseconds per run of one candidate: one warm-up, then `reps` runs between two events
    auto time_config = [&](const patdnn_config_t& c, int reps, float& ms) -> patdnn_status_t {
        patdnn_status_t r = run_config(h, c, s, input, bias, output, stream, workspace, workspace_floats);
        if (r != PATDNN_OK) return r;
        (void)hipEventRecord(e0, stream);
        for (int k = 0; k < reps && r == PATDNN_OK; ++k)
            r = run_config(h, c, s, input, bias, output, stream, workspace, workspace_floats);
        (void)hipEventRecord(e1, stream);
        if (r != PATDNN_OK) return r;
        hipError_t he = hipEventSynchronize(e1);
        if (he != hipSuccess) return hip_fail(he, "hipEventSynchronize");
        ms = 0.0f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        ms /= (float)reps;
        return PATDNN_OK;
    };
    // first pass over every candidate, then the four fastest again, in turns (clocks and cache
    // contents drift while a process tunes: a candidate timed later is not timed under the
    // same conditions as one timed earlier), each judged by the median of its turns: the
    // winner of a noisy first pass should not stay by luck
    std::vector<std::pair<float, size_t>> timed;
    for (size_t i = 0; i < cands.size(); ++i) {
        float ms = 0.0f;
        st = time_config(cands[i], 3, ms);
        if (st != PATDNN_OK) { result = st; break; }
        timed.emplace_back(ms, i);
    }
    if (result == PATDNN_OK) {
        std::sort(timed.begin(), timed.end());
        const size_t finalists = std::min<size_t>(timed.size(), 4);
        constexpr int kTurns = 5;
        std::vector<std::vector<float>> turns(finalists);
        for (int t = 0; t < kTurns && result == PATDNN_OK; ++t)
            for (size_t k = 0; k < finalists; ++k) {
                float ms = 0.0f;
                st = time_config(cands[timed[k].second], 3, ms);
                if (st != PATDNN_OK) { result = st; break; }
                turns[k].push_back(ms);
            }
        for (size_t k = 0; k < finalists && result == PATDNN_OK; ++k) {
            std::sort(turns[k].begin(), turns[k].end());
            const float ms = turns[k][turns[k].size() / 2];
            if (best < 0.0f || ms < best) { best = ms; best_cfg = cands[timed[k].second]; }
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (result != PATDNN_OK) return result;
    // leave a valid result of the chosen configuration in `output`
    st = run_config(h, best_cfg, s, input, bias, output, stream, workspace, workspace_floats);
    if (st != PATDNN_OK) return st;
    if ((e = hipStreamSynchronize(stream)) != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    h->cfg = best_cfg;
    h->cfg_tuned = true;
    // keep the winner's layout and the default variant's; free the others
    {
        const patdnn_config_t dflt = default_config(h, s);
        for (auto it = h->tiled.begin(); it != h->tiled.end();) {
            const int vnum = it->first.first + 1;
            const bool dense = tiled_variant(it->first.first).dense;
            const bool keep = (vnum == best_cfg.variant && (dense || it->first.second == best_cfg.ck)) ||
                              (vnum == dflt.variant && (dense || it->first.second == dflt.ck));
            it = keep ? std::next(it) : h->tiled.erase(it);
        }
    }
    if (best_us) *best_us = best * 1000.0f;
    return PATDNN_OK;
}

static patdnn_status_t find_tiled(patdnn_handle_t h, int32_t variant, int32_t ck, TiledOnDevice** out)
{
    if (!h) return fail(PATDNN_EINVAL, "handle is NULL");
    const int vi = variant - 1;
    if (extra_variant(variant) >= 0 && variant < patdnn_num_variants())
        return fail(PATDNN_EUNSUPPORTED, "this variant has no filter-group layout");
    if (vi < 0 || vi >= num_tiled_variants()) return fail(PATDNN_EINVAL, "not a tiled variant");
    const TiledVariant& v = tiled_variant(vi);
    if (v.dense || !variant_fits_layer(h, v)) return fail(PATDNN_EUNSUPPORTED, "variant cannot run this layer");
    if (ck < 0) return fail(PATDNN_EINVAL, "ck out of range");
    if (ck == 0) ck = default_ck(v, h->L.desc.c_in);
    ck = std::min(ck, h->L.desc.c_in);
    if (ck * 4 * v.lds_buffers * v.lds_floats_per_channel > kMaxLdsBytes) return fail(PATDNN_EUNSUPPORTED, "ck exceeds the LDS budget");
    try {
        patdnn_status_t st = ensure_tiled(h, vi, ck, nullptr);
        if (st != PATDNN_OK) return st;
    } catch (const std::bad_alloc&) {
        return fail(PATDNN_ENOMEM, "out of host memory");
    }
    *out = h->tiled.find(std::make_pair(vi, ck))->second.get();
    return PATDNN_OK;
}

patdnn_status_t patdnn_tiled_info(patdnn_handle_t h, int32_t variant, int32_t ck, patdnn_tiled_info_t* out)
{
    if (!out) return fail(PATDNN_EINVAL, "out is NULL");
    TiledOnDevice* t = nullptr;
    patdnn_status_t st = find_tiled(h, variant, ck, &t);
    if (st != PATDNN_OK) return st;
    const TiledVariant& v = tiled_variant(variant - 1);
    out->G = t->host.G;
    out->num_groups = t->host.num_groups;
    out->ck = t->host.ck;
    out->num_chunks = t->host.num_chunks;
    out->num_steps = (int64_t)(t->host.steps.size() / kStepDwords);
    out->block_bytes = v.block_bytes;
    out->table_off = v.table_off;
    out->ctrl_bytes = v.ctrl_bytes;
    out->records = v.records;
    out->double_window = v.double_window ? 1 : 0;
    out->lds_channel_bytes = 4 * v.lds_floats_per_channel;
    out->threaded = v.threaded ? 1 : 0;
    out->patch_rows = v.PR;
    out->patch_cols = v.PC;
    out->conv_stride = v.S;
    out->lanes_x = v.TGX;
    out->experimental = v.experimental ? 1 : 0;
    out->mode = v.mode;
    return PATDNN_OK;
}

patdnn_status_t patdnn_export_tiled(patdnn_handle_t h, int32_t variant, int32_t ck,
                                    int32_t* slot_channel, uint32_t* chunk_ptr, uint32_t* steps)
{
    TiledOnDevice* t = nullptr;
    patdnn_status_t st = find_tiled(h, variant, ck, &t);
    if (st != PATDNN_OK) return st;
    auto get = [&](void* dst, const void* dev, const void* host, size_t bytes) -> hipError_t {
        if (!dst || !bytes) return hipSuccess;
        if (h->on_device) return hipMemcpy(dst, dev, bytes, hipMemcpyDeviceToHost);
        std::memcpy(dst, host, bytes);
        return hipSuccess;
    };
    hipError_t e;
    if ((e = get(slot_channel, t->dev.slot_channel, t->host.slot_channel.data(), t->host.slot_channel.size() * 4)) != hipSuccess ||
        (e = get(chunk_ptr, t->dev.chunk_ptr, t->host.chunk_ptr.data(), t->host.chunk_ptr.size() * 4)) != hipSuccess ||
        (e = get(steps, t->dev.steps, t->host.steps.data(), t->host.steps.size() * 4)) != hipSuccess)
        return hip_fail(e, "reading the tiled layout back");
    return PATDNN_OK;
}

patdnn_status_t patdnn_selftest(void)
{
    std::string why;
    if (!movrel_selftest(why)) return fail(PATDNN_EUNSUPPORTED, why);
    return PATDNN_OK;
}

void patdnn_destroy(patdnn_handle_t h) { delete h; }

// ---------------------------------------------------------------------------
// A stack of layers run back to back (section 6.2: one image through all CONV layers)
// ---------------------------------------------------------------------------
}  // extern "C"

struct patdnn_stack {
    std::vector<patdnn_stack_layer_t> layers;
    int32_t n = 0;
    std::vector<int32_t> in_h, in_w;          // input size of every layer
    int32_t out_shape[4] = {0, 0, 0, 0};
    size_t max_intermediate = 0;              // floats of the largest tensor between two layers
    size_t buf_floats[2] = {0, 0};            // floats the tensors written to buffer 0 / 1 need
    size_t split_floats_min = 0;              // largest un-pooled output of a pooled layer (partial sums)
    size_t split_floats = 0;                  // >= split_floats_min: room for one buffer per channel slice
    float* buf[2] = {nullptr, nullptr};       // the stack's own ping-pong buffers
    float* split = nullptr;                   // and its buffer for the partial sums of split pooled layers
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    const float* graph_in = nullptr;
    float* graph_out = nullptr;
    bool warmed = false;                      // one plain run has set every function attribute

    ~patdnn_stack()
    {
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
        for (float* p : buf)
            if (p) (void)hipFree(p);
        if (split) (void)hipFree(split);
    }
};

namespace {

// A stack gives its split layers one partial-sum buffer per channel slice up to this size
// (512 MB); a layer that would need more adds its slices up with atomics instead.
constexpr size_t kMaxSliceFloats = (size_t)128 << 20;

// every layer on `stream`, intermediates alternating between b0 and b1
patdnn_status_t stack_launch(patdnn_stack* s, const float* input, float* output, float* b0, float* b1,
                             float* split, size_t split_floats, hipStream_t stream)
{
    const int L = (int)s->layers.size();
    auto dst_of = [&](int i) { return i == L - 1 ? output : ((i & 1) ? b1 : b0); };
    const float* src = input;
    // A layer that ends with a finishing kernel (its input channels are split) clears there what
    // the next layer adds into, which saves that layer a fill launch of its own: some 5 us each,
    // a tenth of a single image's latency.  The region is the next layer's output (the buffer this
    // layer has just finished reading) or the partial-sum buffer, never what this layer itself
    // still reads or writes (the launcher checks the one case that could coincide).
    ZeroRegion zeroed;
    for (int i = 0; i < L; ++i) {
        float* dst = dst_of(i);
        const patdnn_stack_layer_t& ly = s->layers[i];
        ZeroHandoff hand;
        hand.pre_zeroed = zeroed;
        if (i + 1 < L) {
            const patdnn_stack_layer_t& nx = s->layers[i + 1];
            hand.next = zero_need(nx.layer, s->n, s->in_h[i + 1], s->in_w[i + 1], nx.pool2, dst_of(i + 1), split,
                                  split_floats);
            if (hand.next.p == dst) hand.next = ZeroRegion{};     // this layer's own output: cannot happen
        }
        patdnn_status_t st = conv2d_impl(ly.layer, src, s->n, s->in_h[i], s->in_w[i], ly.bias, dst, ly.fuse_relu,
                                         ly.pool2, stream, split, split_floats, &hand);
        if (st != PATDNN_OK) return st;
        zeroed = hand.done ? hand.next : ZeroRegion{};
        src = dst;
    }
    return PATDNN_OK;
}

}  // namespace

extern "C" {

patdnn_status_t patdnn_stack_create(const patdnn_stack_layer_t* layers, int32_t num_layers, int32_t n,
                                    int32_t h_in, int32_t w_in, patdnn_stack_t* out)
{
    if (out) *out = nullptr;
    if (!layers || !out || num_layers <= 0 || n <= 0) return fail(PATDNN_EINVAL, "layers / out is NULL or a size is not positive");
    std::unique_ptr<patdnn_stack> s(new (std::nothrow) patdnn_stack());
    if (!s) return fail(PATDNN_ENOMEM, "out of host memory");
    s->n = n;
    int32_t h = h_in, w = w_in, c = -1;
    for (int i = 0; i < num_layers; ++i) {
        const patdnn_stack_layer_t& ly = layers[i];
        if (!ly.layer) return fail(PATDNN_EINVAL, "a layer handle is NULL");
        if (!ly.layer->on_device) return fail(PATDNN_EHIP, "a layer was encoded with PATDNN_HOST_ONLY");
        if (c >= 0 && ly.layer->L.desc.c_in != c) return fail(PATDNN_EINVAL, "channel counts of consecutive layers do not match");
        if (ly.pool2 && ly.layer->L.depthwise) return fail(PATDNN_EUNSUPPORTED, "fused pooling is not built for depthwise layers");
        ConvShape cs{};
        patdnn_status_t st = shape_of(ly.layer, n, h, w, cs);
        if (st != PATDNN_OK) return st;
        s->in_h.push_back(h);
        s->in_w.push_back(w);
        h = ly.pool2 ? cs.ho / 2 : cs.ho;
        w = ly.pool2 ? cs.wo / 2 : cs.wo;
        if (h <= 0 || w <= 0) return fail(PATDNN_EINVAL, "a layer's output is empty");
        c = cs.c_out;
        const size_t full = (size_t)n * c * cs.ho * cs.wo;
        if (ly.pool2) s->split_floats_min = std::max(s->split_floats_min, full);
        // one buffer per channel slice for the layers that are configured to split now (a layer
        // reconfigured later uses the room there is, or adds its slices up with atomics)
        const patdnn_config_t& cfg = ly.layer->cfg;
        if (cfg.variant > 0 && cfg.ksplit > 1) {
            const size_t want = (size_t)cfg.ksplit * split_slice_stride(full);
            if (want <= kMaxSliceFloats) s->split_floats = std::max(s->split_floats, want);
        }
        if (i + 1 < num_layers) {
            s->max_intermediate = std::max(s->max_intermediate, (size_t)n * c * h * w);
            s->buf_floats[i & 1] = std::max(s->buf_floats[i & 1], (size_t)n * c * h * w);
        }
        s->layers.push_back(ly);
    }
    s->out_shape[0] = n; s->out_shape[1] = c; s->out_shape[2] = h; s->out_shape[3] = w;
    s->split_floats = std::max(s->split_floats, s->split_floats_min);
    for (int k = 0; k < 2; ++k)
        if (s->buf_floats[k]) {
            hipError_t e = hipMalloc(reinterpret_cast<void**>(&s->buf[k]), s->buf_floats[k] * sizeof(float));
            if (e != hipSuccess) return hip_fail(e, "allocating the stack's intermediate tensors");
        }
    if (s->split_floats) {
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&s->split), s->split_floats * sizeof(float));
        if (e != hipSuccess) return hip_fail(e, "allocating the stack's partial-sum buffer");
    }
    *out = s.release();
    return PATDNN_OK;
}

patdnn_status_t patdnn_stack_output_shape(patdnn_stack_t s, int32_t out_nchw[4])
{
    if (!s || !out_nchw) return fail(PATDNN_EINVAL, "stack / out_nchw is NULL");
    for (int i = 0; i < 4; ++i) out_nchw[i] = s->out_shape[i];
    return PATDNN_OK;
}

patdnn_status_t patdnn_stack_run(patdnn_stack_t s, const float* input, float* output, int32_t use_graph,
                                 void* stream_)
{
    if (!s) return fail(PATDNN_EINVAL, "stack is NULL");
    if (!input || !output) return fail(PATDNN_EINVAL, "input / output is NULL");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (!use_graph) {
        patdnn_status_t st = stack_launch(s, input, output, s->buf[0], s->buf[1], s->split, s->split_floats, stream);
        if (st == PATDNN_OK) s->warmed = true;
        return st;
    }
    if (!stream) return fail(PATDNN_EINVAL, "graph execution needs a stream other than the default one");
    if (!s->exec || s->graph_in != input || s->graph_out != output) {
        // (re)capture: the graph holds the tensor addresses it was recorded with
        if (!s->warmed) {
            // a first plain run sets the per-kernel attributes, which must not happen in a capture
            patdnn_status_t st = stack_launch(s, input, output, s->buf[0], s->buf[1], s->split, s->split_floats, stream);
            if (st != PATDNN_OK) return st;
            s->warmed = true;
        }
        if (s->exec) { (void)hipGraphExecDestroy(s->exec); s->exec = nullptr; }
        if (s->graph) { (void)hipGraphDestroy(s->graph); s->graph = nullptr; }
        hipError_t e = hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal);
        if (e != hipSuccess) return hip_fail(e, "hipStreamBeginCapture");
        patdnn_status_t st = stack_launch(s, input, output, s->buf[0], s->buf[1], s->split, s->split_floats, stream);
        e = hipStreamEndCapture(stream, &s->graph);
        if (st != PATDNN_OK) {
            if (s->graph) { (void)hipGraphDestroy(s->graph); s->graph = nullptr; }
            return st;
        }
        if (e != hipSuccess) return hip_fail(e, "hipStreamEndCapture");
        e = hipGraphInstantiate(&s->exec, s->graph, nullptr, nullptr, 0);
        if (e != hipSuccess) return hip_fail(e, "hipGraphInstantiate");
        s->graph_in = input;
        s->graph_out = output;
    }
    hipError_t e = hipGraphLaunch(s->exec, stream);
    return e == hipSuccess ? PATDNN_OK : hip_fail(e, "hipGraphLaunch");
}

void patdnn_stack_destroy(patdnn_stack_t s) { delete s; }

}  // extern "C"

// ---------------------------------------------------------------------------
// patdnn_stack_run without any allocation behind it: the tensors between the layers and the
// partial sums of split pooled layers live in one file-scope device array instead of the
// stack's own buffers.  Every GPU the library runs on holds its own copy of the array until
// the process ends; calls that overlap on one GPU share it and race.
// ---------------------------------------------------------------------------
namespace {

constexpr size_t kStaticScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];              // device address of `scratch`, per device
std::mutex g_scratch_lock;

// The array's device address on the current device (looked up once per device; in host code
// the array's name is only a handle for this lookup, never an address to pass to a kernel).
hipError_t static_scratch(unsigned char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
    return hipSuccess;
}

size_t round256(size_t bytes) { return (bytes + 255) / 256 * 256; }

}  // namespace

extern "C" {

patdnn_status_t patdnn_stack_run_static(patdnn_stack_t s, const float* input, float* output, void* stream)
{
    if (!s) return fail(PATDNN_EINVAL, "stack is NULL");
    if (!input || !output) return fail(PATDNN_EINVAL, "input / output is NULL");
    const size_t b0 = round256(s->buf_floats[0] * sizeof(float)), b1 = round256(s->buf_floats[1] * sizeof(float));
    // room for one partial-sum buffer per channel slice if the built-in buffer has it, else
    // the one buffer that split pooled layers cannot do without
    size_t sp_floats = s->split_floats;
    if (b0 + b1 + round256(sp_floats * sizeof(float)) > kStaticScratchBytes) sp_floats = s->split_floats_min;
    const size_t sp = round256(sp_floats * sizeof(float));
    if (b0 + b1 + sp > kStaticScratchBytes) {
        char msg[200];
        snprintf(msg, sizeof(msg), "the stack needs %zu bytes between its layers; the built-in buffer of "
                 "patdnn_stack_run_static holds %zu", b0 + b1 + sp, kStaticScratchBytes);
        return fail(PATDNN_EUNSUPPORTED, msg);
    }
    unsigned char* base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return hip_fail(e, "looking up the built-in buffer");
    // nothing here needs to start at zero: the kernels clear the pooled outputs and partial
    // sums they accumulate into, whatever an earlier call left behind
    return stack_launch(s, input, output, reinterpret_cast<float*>(base), reinterpret_cast<float*>(base + b0),
                        reinterpret_cast<float*>(base + b0 + b1), sp_floats, static_cast<hipStream_t>(stream));
}

const char* patdnn_status_string(patdnn_status_t s)
{
    switch (s) {
        case PATDNN_OK: return "ok";
        case PATDNN_EINVAL: return "invalid argument";
        case PATDNN_EPATTERN: return "pattern constraint violated";
        case PATDNN_ENOMEM: return "out of host memory";
        case PATDNN_EHIP: return "HIP runtime error";
        case PATDNN_EUNSUPPORTED: return "unsupported";
    }
    return "unknown status";
}

const char* patdnn_last_error(void) { return g_err.c_str(); }

}  // extern "C"
