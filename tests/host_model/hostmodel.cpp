// Host build of csrc/kernel_tiled.hip - TEST INFRASTRUCTURE (see hip/hip_runtime.h here).
#include <hip/hip_runtime.h>

thread_local dim3 threadIdx;
dim3 blockIdx, blockDim, gridDim;
namespace patdnn { float lds[hostmodel::kLdsFloats]; }

namespace hostmodel {

State& state()
{
    static State s;
    return s;
}

void fail(const char* what, long a, long b)
{
    State& st = state();
    pthread_mutex_lock(&st.lock);
    if (st.errors++ == 0) st.first_error = std::string(what) + " (" + std::to_string(a) + ", " + std::to_string(b) + ")";
    pthread_mutex_unlock(&st.lock);
}

static float lds_read(unsigned byte_addr)
{
    State& st = state();
    const unsigned base = (unsigned)(uintptr_t)patdnn::lds;
    const unsigned rel = byte_addr - base;
    if (rel % 4 || rel / 4 >= st.lds_floats) {
        fail("window read outside the launch's LDS", rel, (long)st.lds_floats);
        return 0.0f;
    }
    return patdnn::lds[rel / 4];
}

}  // namespace hostmodel

// Same semantics as the generated assembly: steps fetched in order, a window register
// set per loaded channel, FMAs in tap-major order.
void hostmodel_walk(const HostmodelGeo& g, float* acc, unsigned lane_lds, const uint32_t* stream,
                    unsigned entry)
{
    using namespace hostmodel;
    const int nwin = g.WR * g.WC, nacc = g.PR * g.PC;
    std::vector<float> win((size_t)2 * nwin, NAN);
    static const int others[8] = {0, 1, 2, 3, 5, 6, 7, 8};
    auto taps_of = [&](int u, int taps[4]) {
        int k = 0;
        for (int a = 0; a < 8; ++a)
            for (int b = a + 1; b < 8; ++b)
                for (int c = b + 1; c < 8; ++c, ++k)
                    if (k == u) {
                        int t[4] = {others[a], others[b], others[c], 4};
                        std::sort(t, t + 4);
                        std::copy(t, t + 4, taps);
                    }
    };
    auto load_window = [&](int set, unsigned off) {
        for (int q = 0; q < g.WR; ++q)
            for (int r = 0; r < g.WC; ++r)
                win[(size_t)set * nwin + q * g.WC + r] = lds_read(lane_lds + off + 4u * (unsigned)(q * g.rowp + r));
    };
    auto kernel = [&](unsigned target, const uint32_t* w4) -> bool {
        if (target < g.table_off || (target - g.table_off) % g.block_bytes) {
            fail("code offset is not a block start", target);
            return false;
        }
        const unsigned idx = (target - g.table_off) / g.block_bytes;
        const int set = (int)(idx / (unsigned)(g.G * 56)), rest = (int)(idx % (unsigned)(g.G * 56));
        const int slot = rest / 56, u = rest % 56;
        if (set >= g.sets) { fail("window set out of range", set); return false; }
        int taps[4];
        taps_of(u, taps);
        for (int t = 0; t < 4; ++t) {
            float wv;
            std::memcpy(&wv, &w4[t], 4);
            const int kh = taps[t] / 3, kw = taps[t] % 3;
            for (int r = 0; r < g.PR; ++r)
                for (int c = 0; c < g.PC; ++c) {
                    float& a = acc[slot * nacc + r * g.PC + c];
                    a = fmaf(wv, win[(size_t)set * nwin + (r * g.S + kh) * g.WC + c * g.S + kw], a);
                }
        }
        return true;
    };
    const unsigned cb = g.ctrl_bytes;
    for (long k = 0; k < (1l << 22); ++k) {
        const uint32_t* st = stream + 24 * k;
        if (!g.threaded) {
            const unsigned blk = st[20] / cb;
            if (st[20] % cb || !(blk <= 2 || blk == 5)) { fail("bad window block", st[20]); return; }
            if (blk == 5) return;
            if (blk <= 1) load_window(g.sets == 2 ? (int)blk : 0, st[21]);
            const unsigned done = ((k & 1) ? 4u : 3u) * cb;
            for (unsigned q = 0; q < g.records; ++q) {
                if (st[16 + q] == done) break;
                if (!kernel(st[16 + q], st + 4 * q)) return;
            }
        } else {
            if (entry % cb || entry / cb > 6) { fail("bad step entry", entry); return; }
            const unsigned e = entry / cb;
            if (e == 6) return;
            if ((e / 3) != (unsigned)(k & 1)) { fail("step entered through the other register set", e, k); return; }
            if (e % 3) load_window(g.sets == 2 ? (int)(e % 3) - 1 : 0, st[23]);
            unsigned q = 0;
            for (;; ++q) {
                const unsigned tg = q < g.records ? st[6 * q + 4] : st[22];
                if (tg < g.table_off) { entry = tg; break; }
                if (q >= g.records) { fail("step has no end"); return; }
                if (!kernel(tg, st + 6 * q)) return;
            }
        }
    }
    fail("stream does not end");
}

#include "kernel_tiled.hip"

extern "C" {

// Runs one tiled variant on host arrays; returns the number of violations (0 = clean) and
// copies the first message into `msg`.
long hostmodel_run(int variant, int G, int num_groups, int ck, int num_chunks, const int32_t* slot_channel,
                   const uint32_t* chunk_ptr, const uint32_t* steps, const float* w9, int n, int c_in, int c_out,
                   int h, int w, int ho, int wo, int stride, int pad, int relu, const float* in,
                   const float* bias, float* out, int waves, int ksplit, float* scratch, size_t scratch_floats,
                   char* msg, int msg_len)
{
    using namespace patdnn;
    hostmodel::State& st = hostmodel::state();
    st.errors = 0;
    st.first_error.clear();
    st.in = in;
    st.in_floats = (size_t)n * c_in * h * w;
    st.out = out;
    st.out_floats = (size_t)n * c_out * ho * wo;
    if (variant < 0 || variant >= num_tiled_variants()) return -1;
    DevTiled t;
    t.G = G; t.num_groups = num_groups; t.ck = ck; t.num_chunks = num_chunks;
    t.slot_channel = slot_channel; t.chunk_ptr = chunk_ptr; t.steps = steps; t.w9 = w9;
    ConvShape s{n, c_in, c_out, h, w, ho, wo, stride, pad, relu};
    const hipError_t e = tiled_variant(variant).launch(t, s, in, bias, out, waves, ksplit, scratch, scratch_floats, nullptr);
    if (e != hipSuccess) hostmodel::fail("launch refused", e);
    if (msg && msg_len > 0) {
        std::strncpy(msg, st.first_error.c_str(), (size_t)msg_len - 1);
        msg[msg_len - 1] = 0;
    }
    return st.errors;
}

// The kernel's division by a launch-time constant, as the launcher sets it up.
unsigned hostmodel_fast_div(unsigned n, unsigned d) { return patdnn::fast_div(n, patdnn::make_fast_div(d)); }

int hostmodel_variant_lds_floats(int variant) { return patdnn::tiled_variant(variant).lds_floats_per_channel; }
int hostmodel_variant_max_slots(int variant) { return patdnn::tiled_variant(variant).max_slots; }

}  // extern "C"
