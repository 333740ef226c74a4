// Offline stage: validation, filter-kernel reorder (paper section 5.2), FKW compact
// storage (section 5.3) and the channel-major filter-group layout of the tiled
// kernels.  Pure host code; no HIP calls.
#include "layout.hpp"

#include <algorithm>
#include <cstring>
#include <numeric>

namespace patdnn {

int universe_index(uint16_t mask)
{
    for (int i = 0; i < kUniverse; ++i)
        if (universe_mask(i) == mask) return i;
    return -1;
}

static int popcount16(unsigned v)
{
    int c = 0;
    for (; v; v &= v - 1) ++c;
    return c;
}

patdnn_status_t build_fkw(const patdnn_layer_desc_t& d, const float* w, const uint8_t* ids,
                          const uint8_t* mask, LayerHost& L, std::string& err)
{
    if (!w) { err = "dense_weights is NULL"; return PATDNN_EINVAL; }
    if (d.c_out <= 0 || d.c_in <= 0) { err = "c_out and c_in must be positive"; return PATDNN_EINVAL; }
    if (d.stride != 1 && d.stride != 2) { err = "stride must be 1 or 2"; return PATDNN_EINVAL; }
    if (d.pad != 0 && d.pad != 1) { err = "pad must be 0 or 1"; return PATDNN_EINVAL; }
    const bool depthwise = d.groups != 1;
    if (d.groups != 1 && !(d.groups == d.c_in && d.c_in == d.c_out)) {
        err = "groups must be 1, or equal to c_in == c_out (depthwise)";
        return PATDNN_EINVAL;
    }
    const bool dense = (d.flags & PATDNN_DENSE) != 0;
    const int kpf = depthwise ? 1 : d.c_in;          // kernels per filter
    const int P = dense ? 1 : d.num_patterns;

    L.desc = d;
    L.desc.pattern_masks = nullptr;
    L.depthwise = depthwise;
    L.dense = dense;
    L.all_in_universe = true;
    Fkw& f = L.fkw;
    f = Fkw();
    f.taps = dense ? 9 : 4;
    f.num_patterns = P;

    if (dense) {
        f.masks.assign(1, 0x1FF);
        L.universe_of_pattern.assign(1, 255);
    } else {
        if (d.num_patterns < 1 || d.num_patterns > 255) {
            err = "num_patterns must be in 1..255";
            return PATDNN_EINVAL;
        }
        if (!d.pattern_masks || !ids) { err = "pattern_masks / pattern_ids is NULL"; return PATDNN_EINVAL; }
        f.masks.assign(d.pattern_masks, d.pattern_masks + P);
        L.universe_of_pattern.resize(P);
        for (int p = 0; p < P; ++p) {
            if (f.masks[p] >= 512 || popcount16(f.masks[p]) != 4) {
                err = "pattern mask " + std::to_string(p) + " does not keep exactly 4 of the 9 positions";
                return PATDNN_EPATTERN;
            }
            const int u = universe_index(f.masks[p]);
            L.universe_of_pattern[p] = (uint8_t)(u < 0 ? 255 : u);
            if (u < 0) L.all_in_universe = false;
        }
    }

    auto kept_at = [&](int co, int k) -> bool {
        return dense || !mask || mask[(size_t)co * kpf + k] != 0;
    };

    // validation of ids (kept kernels only) and, if asked, of the zero structure
    for (int co = 0; co < d.c_out; ++co)
        for (int k = 0; k < kpf; ++k) {
            const size_t kid = (size_t)co * kpf + k;
            const bool kept = kept_at(co, k);
            if (kept && !dense && ids[kid] >= P) {
                err = "pattern id out of range at filter " + std::to_string(co) + ", kernel " + std::to_string(k);
                return PATDNN_EPATTERN;
            }
            if (d.flags & PATDNN_STRICT) {
                const unsigned m = !kept ? 0u : f.masks[dense ? 0 : ids[kid]];
                for (int p = 0; p < 9; ++p)
                    if (!((m >> p) & 1u) && w[kid * 9 + p] != 0.0f) {
                        err = "non-zero weight outside the pattern at filter " + std::to_string(co) +
                              ", kernel " + std::to_string(k);
                        return PATDNN_EPATTERN;
                    }
            }
        }

    // ---- filter reorder: by length, then by per-pattern kernel counts, then by index
    std::vector<int32_t> length(d.c_out, 0);
    std::vector<int32_t> counts((size_t)d.c_out * P, 0);
    for (int co = 0; co < d.c_out; ++co)
        for (int k = 0; k < kpf; ++k)
            if (kept_at(co, k)) {
                ++length[co];
                ++counts[(size_t)co * P + (dense ? 0 : ids[(size_t)co * kpf + k])];
            }
    std::vector<int32_t> order(d.c_out);
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int a, int b) {
        if (length[a] != length[b]) return length[a] < length[b];
        const int32_t* ca = &counts[(size_t)a * P];
        const int32_t* cb = &counts[(size_t)b * P];
        for (int p = 0; p < P; ++p)
            if (ca[p] != cb[p]) return ca[p] < cb[p];
        return a < b;
    });

    // ---- kernel reorder + the five arrays
    int64_t kept_total = 0;
    for (int co = 0; co < d.c_out; ++co) kept_total += length[co];
    if (kept_total > INT32_MAX / 16) { err = "layer too large"; return PATDNN_EUNSUPPORTED; }
    L.kept = kept_total;
    f.offset.assign(d.c_out + 1, 0);
    f.reorder.assign(order.begin(), order.end());
    f.stride.assign((size_t)d.c_out * (P + 1), 0);
    f.index.resize(kept_total);
    f.weight.resize((size_t)kept_total * f.taps);
    int32_t pos = 0;
    for (int s = 0; s < d.c_out; ++s) {
        const int co = order[s];
        f.offset[s] = pos;
        int32_t* st = &f.stride[(size_t)s * (P + 1)];
        for (int p = 0; p < P; ++p) {
            st[p] = pos - f.offset[s];
            for (int k = 0; k < kpf; ++k) {          // ascending input channel inside a pattern
                const size_t kid = (size_t)co * kpf + k;
                if (!kept_at(co, k)) continue;
                if (!dense && ids[kid] != p) continue;
                f.index[pos] = depthwise ? co : k;
                const unsigned m = f.masks[p];
                float* dst = &f.weight[(size_t)pos * f.taps];
                int t = 0;
                for (int q = 0; q < 9; ++q)
                    if ((m >> q) & 1u) dst[t++] = w[kid * 9 + q];
                ++pos;
            }
        }
        st[P] = pos - f.offset[s];
    }
    f.offset[d.c_out] = pos;
    return PATDNN_OK;
}

void decode_fkw(const LayerHost& L, const Fkw& f, float* w, uint8_t* ids, uint8_t* mask)
{
    const int c_out = L.desc.c_out;
    const int kpf = L.depthwise ? 1 : L.desc.c_in;
    const int P = f.num_patterns;
    const size_t nk = (size_t)c_out * kpf;
    if (w) std::memset(w, 0, nk * 9 * sizeof(float));
    if (ids) std::memset(ids, 0, nk);
    if (mask) std::memset(mask, 0, nk);
    for (int s = 0; s < c_out; ++s) {
        const int co = f.reorder[s];
        const int32_t* st = &f.stride[(size_t)s * (P + 1)];
        for (int p = 0; p < P; ++p)
            for (int32_t k = f.offset[s] + st[p]; k < f.offset[s] + st[p + 1]; ++k) {
                const int kk = L.depthwise ? 0 : f.index[k];
                const size_t kid = (size_t)co * kpf + kk;
                if (mask) mask[kid] = 1;
                if (ids) ids[kid] = L.dense ? 0 : (uint8_t)p;
                if (w) {
                    const unsigned m = f.masks[p];
                    int t = 0;
                    for (int q = 0; q < 9; ++q)
                        if ((m >> q) & 1u) w[kid * 9 + q] = f.weight[(size_t)k * f.taps + t++];
                }
            }
    }
}

void build_tiled(const LayerHost& L, const TiledParams& prm, Tiled& T)
{
    const Fkw& f = L.fkw;
    const int G = prm.G;
    const int c_out = L.desc.c_out, c_in = L.desc.c_in, P = f.num_patterns;
    T = Tiled();
    T.G = G;
    T.dense = L.dense;
    T.num_groups = (c_out + G - 1) / G;
    T.slot_channel.assign((size_t)T.num_groups * G, -1);
    T.group_kernels.assign(T.num_groups, 0);
    if (L.dense) {
        T.w9.assign((size_t)T.num_groups * c_in * G * 9, 0.0f);
    } else {
        T.ck = prm.ck;
        T.num_chunks = (c_in + prm.ck - 1) / prm.ck;
        T.chunk_ptr.assign((size_t)T.num_groups * T.num_chunks, 0);
    }

    struct Entry { uint32_t chan, upat, slot; int32_t k; };
    // one step before it is laid out: its kernels ([first, last) in `ent`), the window
    // register set they read, and the window its entry loads (action 0 none, 1 / 2 set 0 / 1)
    struct Step { size_t first, last; uint32_t set, action, window_off; };
    const uint32_t R = prm.records;
    auto ctrl = [&](int which) { return (uint32_t)which * prm.ctrl_bytes; };
    auto float_bits = [](float v) { uint32_t u; std::memcpy(&u, &v, 4); return u; };
    std::vector<Step> plan;

    // ---- which filters share a group.  The wavefronts of a workgroup (consecutive groups)
    // meet at a barrier after every chunk of input channels, so what has to be equal is the
    // work of the groups chunk by chunk - the purpose the paper's filter reorder serves for
    // the threads of a block (section 5.2).  Filters are dealt out longest first, each to
    // the group with a free slot whose per-chunk load stays flattest (sum of squares), then
    // pairs of filters are swapped between groups while that improves.  Dense layers have
    // equal filters and keep the stored order.
    std::vector<int32_t> members((size_t)T.num_groups * G, -1);    // [group][slot] -> FKW position
    if (L.dense) {
        for (int r = 0; r < c_out; ++r) members[r] = c_out - 1 - r;
    } else {
        const int nc = T.num_chunks, ng = T.num_groups;
        std::vector<int32_t> fc((size_t)c_out * nc, 0);             // kernels of a filter per chunk
        for (int s = 0; s < c_out; ++s)
            for (int32_t k = f.offset[s]; k < f.offset[s + 1]; ++k) ++fc[(size_t)s * nc + f.index[k] / prm.ck];
        std::vector<int64_t> load((size_t)ng * nc, 0);
        std::vector<int32_t> fill(ng, 0);
        auto delta_sq = [&](int g, const int32_t* add, const int32_t* sub) {
            int64_t d = 0;                                           // change of sum(load^2) of group g
            for (int c = 0; c < nc; ++c) {
                const int64_t a = load[(size_t)g * nc + c], b = a + add[c] - (sub ? sub[c] : 0);
                d += b * b - a * a;
            }
            return d;
        };
        for (int r = 0; r < c_out; ++r) {
            const int s = c_out - 1 - r;                             // FKW order ascends in length
            int best = -1;
            int64_t best_d = 0;
            for (int g = 0; g < ng; ++g) {
                if (fill[g] >= G) continue;
                const int64_t d = delta_sq(g, &fc[(size_t)s * nc], nullptr);
                if (best < 0 || d < best_d) { best = g; best_d = d; }
            }
            members[(size_t)best * G + fill[best]++] = s;
            for (int c = 0; c < nc; ++c) load[(size_t)best * nc + c] += fc[(size_t)s * nc + c];
        }
        // bounded improvement by swaps; a fixed linear congruential sequence picks the pairs
        uint64_t lcg = 0x9E3779B97F4A7C15ull;
        const long attempts = std::min<long>(200000, 200l * c_out);
        for (long it = 0; it < attempts && ng > 1; ++it) {
            lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
            const int ia = (int)((lcg >> 33) % (uint64_t)members.size());
            lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
            const int ib = (int)((lcg >> 33) % (uint64_t)members.size());
            const int ga = ia / G, gb = ib / G, sa = members[ia], sb = members[ib];
            if (ga == gb || sa < 0 || sb < 0) continue;
            const int32_t* fa = &fc[(size_t)sa * nc];
            const int32_t* fb = &fc[(size_t)sb * nc];
            if (delta_sq(ga, fb, fa) + delta_sq(gb, fa, fb) >= 0) continue;
            for (int c = 0; c < nc; ++c) {
                load[(size_t)ga * nc + c] += fb[c] - fa[c];
                load[(size_t)gb * nc + c] += fa[c] - fb[c];
            }
            std::swap(members[ia], members[ib]);
        }
    }

    std::vector<Entry> ent;
    for (int g = 0; g < T.num_groups; ++g) {
        ent.clear();
        for (int slot = 0; slot < G; ++slot) {
            const int s = members[(size_t)g * G + slot];   // FKW position of the filter
            if (s < 0) continue;
            T.slot_channel[(size_t)g * G + slot] = f.reorder[s];
            T.group_kernels[g] += f.offset[s + 1] - f.offset[s];
            const int32_t* st = &f.stride[(size_t)s * (P + 1)];
            for (int p = 0; p < P; ++p)
                for (int32_t k = f.offset[s] + st[p]; k < f.offset[s] + st[p + 1]; ++k) {
                    if (L.dense) {
                        float* dst = &T.w9[(((size_t)g * c_in + f.index[k]) * G + slot) * 9];
                        std::memcpy(dst, &f.weight[(size_t)k * 9], 9 * sizeof(float));
                    } else {
                        ent.push_back({(uint32_t)f.index[k], L.universe_of_pattern[p], (uint32_t)slot, k});
                    }
                }
        }
        if (L.dense) continue;
        std::sort(ent.begin(), ent.end(), [](const Entry& a, const Entry& b) {
            if (a.chan != b.chan) return a.chan < b.chan;
            if (a.upat != b.upat) return a.upat < b.upat;
            return a.slot < b.slot;
        });
        size_t e = 0;
        for (int chunk = 0; chunk < T.num_chunks; ++chunk) {
            const uint32_t c_end = (uint32_t)std::min(c_in, (chunk + 1) * prm.ck);
            const size_t e_begin = e;
            while (e < ent.size() && ent[e].chan < c_end) ++e;
            // channels of this chunk on which the group has kernels: [begin, end) in ent
            std::vector<std::pair<size_t, size_t>> runs;
            for (size_t i = e_begin; i < e;) {
                size_t j = i;
                while (j < e && ent[j].chan == ent[i].chan) ++j;
                runs.emplace_back(i, j);
                i = j;
            }
            auto lds_off = [&](size_t run) {
                return (ent[runs[run].first].chan - (uint32_t)chunk * prm.ck) * prm.channel_bytes;
            };
            // ---- the steps of this chunk, independent of how they are dispatched
            plan.clear();
            if (prm.double_window && !runs.empty())
                plan.push_back({0, 0, 0u, 1u, lds_off(0)});          // only loads the first window
            for (size_t r = 0; r < runs.size(); ++r) {
                const uint32_t set = prm.double_window ? (uint32_t)(r & 1) : 0u;
                for (size_t i = runs[r].first; i < runs[r].second; i += R) {
                    Step st{i, std::min(i + R, runs[r].second), set, 0u, 0u};
                    if (i == runs[r].first) {
                        if (!prm.double_window) {
                            st.action = 1;
                            st.window_off = lds_off(r);
                        } else if (r + 1 < runs.size()) {
                            st.action = 1 + (uint32_t)((r + 1) & 1);
                            st.window_off = lds_off(r + 1);
                        }
                    }
                    plan.push_back(st);
                }
            }
            // ---- lay them out
            const size_t first_step = T.steps.size() / kStepDwords;
            if (first_step > kChunkStepMask) { T.steps.clear(); T.overflow = true; return; }
            auto block_of = [&](const Step& st, const Entry& x) {
                return prm.table_off +
                       ((st.set * (uint32_t)G + x.slot) * (uint32_t)kUniverse + x.upat) * prm.block_bytes;
            };
            if (!prm.threaded) {
                T.chunk_ptr[(size_t)g * T.num_chunks + chunk] = (uint32_t)first_step;
                for (size_t k = 0; k <= plan.size(); ++k) {
                    const size_t at = T.steps.size();
                    T.steps.resize(at + kStepDwords, 0u);
                    uint32_t* d = &T.steps[at];
                    const uint32_t done = ctrl((k & 1) ? kCtrlDoneB : kCtrlDoneA);   // odd steps: register set B
                    d[16] = done;
                    if (k == plan.size()) { d[20] = ctrl(kCtrlEnd); break; }
                    const Step& st = plan[k];
                    d[20] = ctrl(st.action == 0 ? kCtrlNone : st.action == 1 ? kCtrlLoadA : kCtrlLoadB);
                    d[21] = st.window_off;
                    const size_t n = st.last - st.first;
                    for (size_t q = 0; q < n; ++q) {
                        const Entry& x = ent[st.first + q];
                        const float* w = &f.weight[(size_t)x.k * 4];
                        for (int t = 0; t < 4; ++t) d[4 * q + t] = float_bits(w[t]);
                        d[16 + q] = block_of(st, x);
                    }
                    if (n < R) d[16 + n] = done;
                }
            } else {
                auto enter = [&](size_t k) {        // control block that enters step k of the chunk
                    return k == plan.size() ? (uint32_t)kThreadedEnd
                                            : (uint32_t)(3 * (k & 1)) + plan[k].action;
                };
                T.chunk_ptr[(size_t)g * T.num_chunks + chunk] =
                    (uint32_t)first_step | (enter(0) << kChunkEntryShift);
                for (size_t k = 0; k < plan.size(); ++k) {
                    const size_t at = T.steps.size();
                    T.steps.resize(at + kStepDwords, 0u);
                    uint32_t* d = &T.steps[at];
                    const Step& st = plan[k];
                    d[kThreadedWoff] = st.window_off;
                    const size_t n = st.last - st.first;
                    for (size_t q = 0; q < n; ++q) {
                        const Entry& x = ent[st.first + q];
                        const float* w = &f.weight[(size_t)x.k * 4];
                        for (int t = 0; t < 4; ++t) d[kThreadedRecDwords * q + t] = float_bits(w[t]);
                        d[kThreadedRecDwords * q + 4] = block_of(st, x);
                    }
                    d[n < R ? kThreadedRecDwords * n + 4 : (size_t)kThreadedTermFull] = ctrl((int)enter(k + 1));
                }
            }
        }
    }
    // the interpreter fetches one step beyond the last one it runs
    if (!L.dense) T.steps.resize(T.steps.size() + kStepDwords, 0u);
}

}  // namespace patdnn
