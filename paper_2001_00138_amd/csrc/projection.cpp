// The projection operators of the pattern-based pruning stage, as host utilities that turn a
// dense weight tensor into the three arrays patdnn_encode takes (declared in include/patdnn.h).
//   natural pattern (paper section 4.1): the centre of a kernel plus its three other
//     largest-magnitude positions; the k most frequent ones form the pattern set.
//   pattern projection (section 4.2, sub-problem 2): per kernel the pattern of the set that
//     retains the largest sum of squares - the Euclidean projection onto the pattern constraint.
//   connectivity projection (section 4.2, sub-problem 3): keep the alpha kernels with the
//     largest L2 norms.
// Magnitudes and norms are compared in double computed from the fp32 weights (sums over
// positions 0..8 in that order); ties go to the lower position, the lower mask value, the
// lower pattern id and the lower kernel index co*c_in + ci respectively.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <map>
#include <new>
#include <numeric>
#include <string>
#include <utility>
#include <vector>

#include "../../include/patdnn.h"

namespace patdnn {
void set_last_error(const std::string& msg);     // patdnn_api.hip
}

namespace {

patdnn_status_t bad(patdnn_status_t s, const char* msg)
{
    patdnn::set_last_error(msg);
    return s;
}

uint16_t natural_pattern(const float* k)
{
    int others[8] = {0, 1, 2, 3, 5, 6, 7, 8};
    std::stable_sort(others, others + 8, [&](int a, int b) {
        return std::fabs((double)k[a]) > std::fabs((double)k[b]);
    });
    return (uint16_t)((1u << 4) | (1u << others[0]) | (1u << others[1]) | (1u << others[2]));
}

double retained(const float* k, unsigned mask)
{
    double e = 0.0;
    for (int p = 0; p < 9; ++p)
        if ((mask >> p) & 1u) e += (double)k[p] * (double)k[p];
    return e;
}

}  // namespace

extern "C" {

patdnn_status_t patdnn_mine_patterns(const float* dense_weights, int32_t c_out, int32_t kernels_per_filter,
                                     int32_t k, uint16_t* pattern_masks, int32_t* found)
{
    if (!dense_weights || !pattern_masks || !found || c_out <= 0 || kernels_per_filter <= 0 || k <= 0)
        return bad(PATDNN_EINVAL, "null pointer or non-positive size");
    try {
        std::map<uint16_t, int64_t> count;
        const size_t nk = (size_t)c_out * kernels_per_filter;
        for (size_t i = 0; i < nk; ++i) ++count[natural_pattern(dense_weights + i * 9)];
        std::vector<std::pair<uint16_t, int64_t>> order(count.begin(), count.end());
        std::sort(order.begin(), order.end(), [](const auto& a, const auto& b) {
            return a.second != b.second ? a.second > b.second : a.first < b.first;
        });
        const int n = (int)std::min<size_t>((size_t)k, order.size());
        for (int i = 0; i < n; ++i) pattern_masks[i] = order[(size_t)i].first;
        *found = n;
    } catch (const std::bad_alloc&) {
        return bad(PATDNN_ENOMEM, "out of host memory");
    }
    return PATDNN_OK;
}

patdnn_status_t patdnn_project_patterns(const float* dense_weights, int32_t c_out, int32_t kernels_per_filter,
                                        const uint16_t* pattern_masks, int32_t num_patterns,
                                        uint8_t* pattern_ids, float* projected)
{
    if (!dense_weights || !pattern_masks || !pattern_ids || c_out <= 0 || kernels_per_filter <= 0)
        return bad(PATDNN_EINVAL, "null pointer or non-positive size");
    if (num_patterns <= 0 || num_patterns > 255) return bad(PATDNN_EINVAL, "num_patterns must be 1..255");
    for (int p = 0; p < num_patterns; ++p)
        if (pattern_masks[p] == 0 || pattern_masks[p] > 0x1FF) return bad(PATDNN_EPATTERN, "a pattern mask is empty or has bits above bit 8");
    const size_t nk = (size_t)c_out * kernels_per_filter;
    for (size_t i = 0; i < nk; ++i) {
        const float* kern = dense_weights + i * 9;
        int best = 0;
        double best_e = -1.0;
        for (int p = 0; p < num_patterns; ++p) {
            const double e = retained(kern, pattern_masks[p]);
            if (e > best_e) { best = p; best_e = e; }
        }
        pattern_ids[i] = (uint8_t)best;
        if (projected)
            for (int p = 0; p < 9; ++p) projected[i * 9 + p] = ((pattern_masks[best] >> p) & 1u) ? kern[p] : 0.0f;
    }
    return PATDNN_OK;
}

patdnn_status_t patdnn_project_connectivity(const float* dense_weights, int32_t c_out, int32_t kernels_per_filter,
                                            int64_t alpha, uint8_t* kernel_mask)
{
    if (!dense_weights || !kernel_mask || c_out <= 0 || kernels_per_filter <= 0 || alpha < 0)
        return bad(PATDNN_EINVAL, "null pointer, non-positive size or negative alpha");
    try {
        const size_t nk = (size_t)c_out * kernels_per_filter;
        std::vector<double> norm(nk);
        for (size_t i = 0; i < nk; ++i) norm[i] = retained(dense_weights + i * 9, 0x1FFu);
        std::vector<size_t> order(nk);
        std::iota(order.begin(), order.end(), (size_t)0);
        const size_t keep = (size_t)std::min<int64_t>(alpha, (int64_t)nk);
        auto before = [&](size_t a, size_t b) { return norm[a] != norm[b] ? norm[a] > norm[b] : a < b; };
        if (keep < nk) std::nth_element(order.begin(), order.begin() + (std::ptrdiff_t)keep, order.end(), before);
        std::fill(kernel_mask, kernel_mask + nk, (uint8_t)0);
        for (size_t i = 0; i < keep; ++i) kernel_mask[order[i]] = 1;
    } catch (const std::bad_alloc&) {
        return bad(PATDNN_ENOMEM, "out of host memory");
    }
    return PATDNN_OK;
}

}  // extern "C"
