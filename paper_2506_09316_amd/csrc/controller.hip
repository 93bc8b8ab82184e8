// Host-side conversion logic of the serving system (paper Section 4.3 "Adaptive Layer-wise Conversion"; the table of
// the trace replay in Section 5.4; the key/value-cache formula of Section 5.3).  No device code: these calls decide
// WHICH layers run as DSLA layers; the kernels of this library then run them.
#include <algorithm>
#include <numeric>
#include <vector>

#include "dsla_internal.h"

extern "C" {

dsla_status dsla_rank_layers(int32_t n_layers, const float *sensitivity, int32_t *order)
{
    if (!sensitivity || !order) return DSLA_ERR_NULL;
    if (n_layers <= 0) return DSLA_ERR_SHAPE;
    for (int32_t i = 0; i < n_layers; ++i)
        if (!(sensitivity[i] == sensitivity[i])) return DSLA_ERR_SHAPE;   // NaN has no rank
    std::iota(order, order + n_layers, 0);
    std::stable_sort(order, order + n_layers, [&](int32_t a, int32_t b) { return sensitivity[a] < sensitivity[b]; });
    return DSLA_OK;
}

float dsla_max_conversion_rate(int64_t prompt_len)
{
    struct Row {
        int64_t below;
        float rate;
    };
    static const Row table[] = {{2048, 0.125f}, {4096, 0.25f}, {8192, 0.375f}};
    for (const Row &r : table)
        if (prompt_len < r.below) return r.rate;
    return 0.5f;
}

int64_t dsla_kv_cache_bytes(int32_t n_layers, int64_t batch, int64_t context, int32_t heads, int32_t d_head,
                            int32_t bytes_per_element)
{
    if (n_layers < 0 || batch < 0 || context < 0 || heads < 0 || d_head < 0 || bytes_per_element < 0) return -1;
    return 2 * static_cast<int64_t>(n_layers) * batch * context * heads * d_head * bytes_per_element;
}

dsla_status dsla_conversion_plan(int32_t n_layers, const int32_t *order, int64_t memory_used, int64_t memory_threshold,
                                 int64_t kv_bytes_per_layer, int64_t state_bytes_per_layer, float max_rate,
                                 uint8_t *converted, int32_t *n_converted, int64_t *memory_after, int32_t *reason)
{
    if (!order || !converted || !n_converted) return DSLA_ERR_NULL;
    if (n_layers <= 0 || !(max_rate >= 0.f && max_rate <= 1.f) || kv_bytes_per_layer < 0 || state_bytes_per_layer < 0)
        return DSLA_ERR_SHAPE;
    std::vector<char> seen(static_cast<size_t>(n_layers), 0);
    for (int32_t i = 0; i < n_layers; ++i) {   // order must be a permutation of the layers
        if (order[i] < 0 || order[i] >= n_layers || seen[order[i]]) return DSLA_ERR_SHAPE;
        seen[order[i]] = 1;
    }
    std::fill(converted, converted + n_layers, static_cast<uint8_t>(0));
    const int32_t cap = static_cast<int32_t>(static_cast<double>(max_rate) * n_layers + 1e-9);
    int64_t used = memory_used;
    int32_t count = 0, why = DSLA_PLAN_NO_PRESSURE;
    if (used > memory_threshold) {
        why = DSLA_PLAN_ALL_CONVERTED;
        for (int32_t i = 0; i < n_layers; ++i) {
            if (count >= cap) {
                why = DSLA_PLAN_QUALITY_LIMIT;
                break;
            }
            converted[order[i]] = 1;
            ++count;
            used += state_bytes_per_layer - kv_bytes_per_layer;
            if (used <= memory_threshold) {
                why = DSLA_PLAN_MEMORY_RELIEF;
                break;
            }
        }
    }
    *n_converted = count;
    if (memory_after) *memory_after = used;
    if (reason) *reason = why;
    return DSLA_OK;
}

}  // extern "C"
