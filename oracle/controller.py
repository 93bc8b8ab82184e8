"""CPU oracle of the host-side conversion logic of the serving system (Section 4.3 "Adaptive Layer-wise
Conversion"): ranking of the layers by sensitivity, the prompt-length table of maximum conversion rates used in the
trace replay (Section 5.4), the key/value-cache size formula (Section 5.3) and the rule that converts layers from
the least sensitive end until memory is relieved or the quality limit stops it.  TEST INFRASTRUCTURE: plain Python,
written from the paper's statements; the product's own implementation is C++ in the library and shares nothing
with this file.
"""


def rank_layers(sensitivity):
    """Section 4.3, "Layer Ranking via Sensitivity": layers in ascending order of sensitivity (the first entry is the
    layer that loses least when converted); equal scores keep the lower layer index first."""
    return [i for _, i in sorted((float(s), i) for i, s in enumerate(sensitivity))]


def max_conversion_rate(prompt_len):
    """Section 5.4, table of the trace replay: the largest fraction of layers converted for a request, by prompt
    length: below 2k tokens 12.5 %, 2k to below 4k 25 %, 4k to below 8k 37.5 %, from 8k 50 % (k = 1024)."""
    if prompt_len < 2048:
        return 0.125
    if prompt_len < 4096:
        return 0.25
    if prompt_len < 8192:
        return 0.375
    return 0.5


def kv_cache_bytes(n_layers, batch, context, heads, d_head, bytes_per_element):
    """Section 5.3: KVCache[B] = 2 * n * b * s * h * d_h * B_byte."""
    return 2 * n_layers * batch * context * heads * d_head * bytes_per_element


def conversion_plan(order, memory_used, memory_threshold, kv_bytes_per_layer, state_bytes_per_layer, max_rate):
    """Section 4.3, "Adaptive Conversion Logic": under memory pressure convert layers from the least sensitive end of
    the queue, each conversion replacing that layer's key/value cache by its fixed-size states, until memory use falls
    to the threshold ("memory relief") or the quality limit - here the cap max_rate on the fraction of layers
    converted, as in the trace replay - stops it ("accuracy at risk").  Returns (converted layer indices in the
    order they were converted, memory use afterwards, reason) with reason in {"no pressure", "memory relief",
    "quality limit", "all converted"}."""
    n = len(order)
    cap = int(max_rate * n + 1e-9)
    converted = []
    used = memory_used
    if used <= memory_threshold:
        return converted, used, "no pressure"
    for layer in order:
        if len(converted) >= cap:
            return converted, used, "quality limit"
        converted.append(layer)
        used += state_bytes_per_layer - kv_bytes_per_layer
        if used <= memory_threshold:
            return converted, used, "memory relief"
    return converted, used, "all converted"
