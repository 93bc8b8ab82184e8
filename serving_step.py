"""The attention layers of a hybrid serving step, as a usage example and a measurement:

    python serving_step.py [--layers 16 --B 8 --T 8192 --decode 128]
    python serving_step.py --hybrid [--layers 32 --B 8 --T 8192 --decode 128]
    python serving_step.py --project [--T 16384 --K 4096]
    python serving_step.py --multi N [--Hkv 8]
    python serving_step.py --packed {equal,pow2,serving,one_long}
    python serving_step.py --entropy [--B 8 --T 8192]
    python serving_step.py --attention-decode [--B 8 --T 8192]
    python serving_step.py --attention-prefill [--B 8 --T 8192]

L layer instances (each with its own blend coefficient and its own pair of states per sequence) prefill a
prompt of T tokens for B sequences and then decode token by token.  The decode step of all layers is captured
into one HIP graph and replayed per token (the library enqueues only kernels and allocates nothing, so it can be
captured); the eager loop is timed beside it.  The decode step of the other half of the stack - as many
softmax-attention layers, each over its own key/value cache of T positions - is timed as well, alone and
interleaved with the DSLA layers.  Inputs are synthetic and shared by the layers: the projections that would produce
them, the prefill of the softmax layers and the MLPs of the stack are not part of this library.
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


# Mixed-length prompt batches for --packed (tokens per request; Llama-2-7B head shape).
MIXES = {
    "equal": [16384] * 4,
    "pow2": [16384] + [8192] * 2 + [4096] * 4 + [2048] * 8,
    "serving": [8192, 6000, 5000, 4100, 3000, 2500, 2048, 1500, 1200, 1000, 800, 600, 512, 300, 200, 100, 64, 33, 7, 1] * 2,
    "one_long": [32768] + [512] * 64,
}


def packed(mix: str, H: int, d: int):
    """Prefill of one packed batch of requests of different lengths (dsla_prefill_varlen); prints one JSON line."""
    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd import binding
    from paper_2506_09316_amd.binding import DSLA_BF16

    lengths = MIXES[mix]
    B, total, mx = len(lengths), sum(lengths), max(lengths)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    rnd = lambda: (torch.randn(total, H, d, device=dev, generator=gen) * d ** -0.5).to(torch.bfloat16)
    gat = lambda: (-torch.nn.functional.softplus(-(torch.randn(total, H, d, device=dev, generator=gen) + 2.0)) / 16.0
                   ).to(torch.bfloat16)
    q, k, v, g1, g2 = rnd(), rnd(), rnd(), gat(), gat()
    o = torch.empty_like(v)
    cu = torch.tensor([0] + list(torch.tensor(lengths).cumsum(0)), dtype=torch.int32, device=dev)
    S1 = torch.zeros(B, H, d, d, device=dev)
    S2 = torch.zeros_like(S1)
    desc = dsla.make_desc(B, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, chunk=64)
    nws = dsla.dsla_prefill_varlen_workspace_bytes(desc, total, mx)
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device=dev)

    def step():
        dsla.dsla_prefill_varlen(desc, total, mx, cu, None, q, k, v, g1, g2, S1, S2, o, ws)

    for _ in range(30):
        step()
    torch.cuda.synchronize()
    binding.profile_enable(True, 4096)
    for _ in range(100):
        step()
    res = binding.profile_collect()
    binding.profile_enable(False, 0)
    kernels = {n: round(1e3 * m / c, 1) for n, (m, c) in res.items() if c}
    us = sum(kernels.values())
    print(json.dumps({"workload": f"packed prefill, mix '{mix}': {B} requests, {total} tokens, longest {mx}, H={H} d={d} bf16",
                      "kernel_us": kernels, "prefill_us": round(us, 1), "tokens_per_s": round(total / us * 1e6, 1),
                      "workspace_MB": round(nws / 1e6, 1)}))


def entropy(B: int, T: int, H: int, d: int):
    """Attention entropy of the final query for one softmax layer's keys (dsla_attention_entropy); one JSON line."""
    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd import binding

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    NSETS = 4   # rotate over several key tensors so that the last-level cache cannot serve them
    ks = [torch.randn(B, T, H, d, device=dev, generator=gen).to(torch.bfloat16) for _ in range(NSETS)]
    q_last = (torch.randn(B, H, d, device=dev, generator=gen) * 1.5).to(torch.bfloat16)
    out = torch.empty(B, H, device=dev)
    nws = dsla.dsla_attention_entropy_workspace_bytes(B, H, d, T)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device=dev)
    for i in range(16):
        dsla.dsla_attention_entropy(q_last, ks[i % NSETS], out, d ** -0.5, ws)
    torch.cuda.synchronize()
    binding.profile_enable(True, 4096)
    for i in range(200):
        dsla.dsla_attention_entropy(q_last, ks[i % NSETS], out, d ** -0.5, ws)
    res = binding.profile_collect()
    binding.profile_enable(False, 0)
    ms, n = res["attention_entropy"]
    us = 1e3 * ms / n
    nbytes = B * T * H * d * 2
    print(json.dumps({"workload": f"attention entropy of the final query: B={B} H={H} d={d} T={T} bf16 keys",
                      "us_per_call": round(us, 2), "key_bytes": nbytes, "GBps": round(nbytes / us / 1e3, 1),
                      "frac_of_8TBps": round(nbytes / us / 1e3 / 8000, 4),
                      "mean_entropy": round(float(out.mean()), 4)}))


def attention_prefill(B: int, T: int, H: int, d: int):
    """The causal softmax prefill of one unconverted layer (dsla_attention_prefill) over a prompt of T tokens; one
    JSON line."""
    import torch
    import paper_2506_09316_amd as dsla

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    rnd = lambda *shape: torch.randn(*shape, device=dev, generator=gen).to(torch.bfloat16)
    q, k, v = rnd(B, T, H, d), rnd(B, T, H, d), rnd(B, T, H, d)
    o = torch.empty_like(v)
    for _ in range(2):
        dsla.dsla_attention_prefill(q, k, v, o, d ** -0.5)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dsla.dsla_attention_prefill(q, k, v, o, d ** -0.5)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    flops = 2.0 * T * T * d * B * H   # Q K^T and P V over the lower triangle
    print(json.dumps({"workload": f"causal softmax prefill of one layer: B={B} H={H} d={d} T={T}, bf16, synthetic inputs",
                      "ms": round(ms, 4), "TFLOPs_causal": round(flops / ms / 1e9, 1),
                      "frac_of_bf16_mfma_peak": round(flops / ms / 1e9 / 2500.0, 4)}))


def attention_decode(B: int, T: int, H: int, d: int):
    """One decode step of an unconverted softmax layer over a cache of T positions (dsla_attention_decode), with the
    DSLA decode step of the same batch beside it; one JSON line."""
    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd import binding
    from paper_2506_09316_amd.binding import DSLA_BF16

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    rnd = lambda *shape: torch.randn(*shape, device=dev, generator=gen).to(torch.bfloat16)
    NSETS = 3   # rotate over several caches so that the last-level cache cannot serve them
    caches = [(rnd(B, T, H, d), rnd(B, T, H, d)) for _ in range(NSETS)]
    q = rnd(B, H, d)
    o = torch.empty_like(q)
    nws = dsla.dsla_attention_decode_workspace_bytes(B, H, d, T)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device=dev)
    # the DSLA step of the same batch
    desc = dsla.make_desc(B, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16)
    states = [(torch.randn(B, H, d, d, device=dev, generator=gen) * 0.1, torch.randn(B, H, d, d, device=dev, generator=gen) * 0.1)
              for _ in range(8)]
    g = (-torch.nn.functional.softplus(-(torch.randn(B, H, d, device=dev, generator=gen) + 2.0)) / 16.0).to(torch.bfloat16)
    kd, vd = rnd(B, H, d), rnd(B, H, d)

    def run(n):
        for i in range(n):
            kc, vc = caches[i % NSETS]
            dsla.dsla_attention_decode(q, kc, vc, o, d ** -0.5, ws)
            s1, s2 = states[i % 8]
            dsla.dsla_decode(desc, q, kd, vd, g, g, s1, s2, o)

    run(12)
    torch.cuda.synchronize()
    binding.profile_enable(True, 4096)
    run(120)
    res = binding.profile_collect()
    binding.profile_enable(False, 0)
    us_attn = 1e3 * res["attention_decode"][0] / res["attention_decode"][1]
    us_dsla = 1e3 * res["decode"][0] / res["decode"][1]
    cache_bytes = 2 * B * T * H * d * 2
    print(json.dumps({"workload": f"decode step of one layer, B={B} H={H} d={d}, context T={T}, bf16",
                      "softmax_attention_us": round(us_attn, 2), "kv_cache_bytes": cache_bytes,
                      "softmax_attention_GBps": round(cache_bytes / us_attn / 1e3, 1),
                      "softmax_attention_frac_of_8TBps": round(cache_bytes / us_attn / 1e3 / 8000, 4),
                      "dsla_decode_us": round(us_dsla, 2), "dsla_state_bytes": B * H * 2 * d * d * 4,
                      "ratio": round(us_attn / us_dsla, 2)}))


def hybrid(n_layers: int, B: int, T: int, H: int, d: int, decode: int):
    """The attention layers of the hybrid serving configuration as one step: a stack of n_layers attention layers of
    which the conversion logic picks the ones that run as DSLA layers (entropy of each layer's final query ->
    ranking -> conversion plan under memory pressure, capped by the prompt-length table), then the prompt through
    every layer (DSLA prefill or causal softmax attention) and `decode` tokens (DSLA decode step or single-query
    attention over the growing cache).  Projections and MLPs are not part of this library; inputs are synthetic and
    shared by the layers.  Prints one JSON line."""
    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd.binding import DSLA_BF16

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609 + 5000)
    rnd = lambda *shape: (torch.randn(*shape, device=dev, generator=gen) * d ** -0.5).to(torch.bfloat16)

    def gates(*shape):
        z = torch.randn(*shape, device=dev, generator=gen) + 2.0
        return (-torch.nn.functional.softplus(-z) / 16.0).to(torch.bfloat16)

    q, k, v, g1, g2 = rnd(B, T, H, d), rnd(B, T, H, d), rnd(B, T, H, d), gates(B, T, H, d), gates(B, T, H, d)
    o = torch.empty_like(v)

    # ---- which layers convert: the library's own signal and logic on synthetic per-layer queries ----
    ent = torch.empty(B, H, device=dev, dtype=torch.float32)
    ews = torch.empty(max(dsla.dsla_attention_entropy_workspace_bytes(B, H, d, T), 16), dtype=torch.uint8, device=dev)
    spread = torch.rand(n_layers, generator=torch.Generator().manual_seed(11)) * 14.0 + 1.0   # peaked .. flat layers
    sens = []
    for l in range(n_layers):
        ql = (q[:, -1].float() * float(spread[l]) * d ** 0.5).to(torch.bfloat16).contiguous()
        dsla.dsla_attention_entropy(ql, k, ent, d ** -0.5, ews)
        sens.append(float(ent.mean().item()))
    order = dsla.dsla_rank_layers(sens)
    kv_layer = dsla.dsla_kv_cache_bytes(1, B, T + decode, H, d, 2)
    state_layer = B * H * 2 * d * d * 4
    rate = dsla.dsla_max_conversion_rate(T)
    used = n_layers * kv_layer
    converted, after, why = dsla.dsla_conversion_plan(order, used, used // 4, kv_layer, state_layer, rate)
    conv = set(converted)

    descs = {l: dsla.make_desc(B, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, gamma=0.2 + 0.6 * (l % 7) / 6.0,
                               chunk=64, zero_init=True) for l in conv}
    S = {l: (torch.empty(B, H, d, d, device=dev), torch.empty(B, H, d, d, device=dev)) for l in conv}
    nws = dsla.dsla_prefill_workspace_bytes(next(iter(descs.values())), T) if conv else 0
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device=dev)
    cap = T + decode
    caches = {l: (rnd(B, cap, H, d), rnd(B, cap, H, d)) for l in range(n_layers) if l not in conv}
    aws = torch.empty(max(dsla.dsla_attention_decode_workspace_bytes(B, H, d, cap), 16), dtype=torch.uint8, device=dev)
    lens = torch.full((B,), T, dtype=torch.int32, device=dev)

    def prefill(layers):
        for l in layers:
            if l in conv:
                dsla.dsla_prefill(descs[l], T, q, k, v, g1, g2, S[l][0], S[l][1], o, ws if nws else None)
            else:
                dsla.dsla_attention_prefill(q, k, v, o, d ** -0.5)

    dq, dk, dv, dg1, dg2 = rnd(B, H, d), rnd(B, H, d), rnd(B, H, d), gates(B, H, d), gates(B, H, d)
    do = torch.empty_like(dv)

    def decode_step(layers):
        for l in layers:
            if l in conv:
                dsla.dsla_decode(descs[l], dq, dk, dv, dg1, dg2, S[l][0], S[l][1], do)
            else:
                dsla.dsla_attention_decode(dq, caches[l][0], caches[l][1], do, d ** -0.5, aws, seq_lens=lens)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    all_layers = list(range(n_layers))
    soft = [l for l in all_layers if l not in conv]
    prefill(all_layers)
    ms_prefill = timed(lambda: prefill(all_layers), 2)
    ms_prefill_dsla = timed(lambda: prefill(sorted(conv)), 2) if conv else 0.0
    ms_prefill_soft = timed(lambda: prefill(soft), 2) if soft else 0.0

    def decode_all():
        for t in range(decode):
            lens.fill_(T + t + 1)
            decode_step(all_layers)

    decode_all()
    ms_decode = timed(decode_all, 1) / decode
    lens.fill_(cap)
    ms_decode_soft_layer = timed(lambda: decode_step(soft[:1]), 20) if soft else 0.0
    ms_decode_dsla_layer = timed(lambda: decode_step(sorted(conv)[:1]), 20) if conv else 0.0
    assert bool(torch.isfinite(o.float()).all()) and bool(torch.isfinite(do.float()).all())
    n_soft = len(soft)
    print(json.dumps({
        "workload": f"attention layers of a hybrid step: {n_layers} layers, B={B} H={H} d={d}, prompt T={T}, {decode} decode "
                    f"tokens, bf16, synthetic inputs; projections and MLPs not included",
        "converted_layers": sorted(conv), "n_converted": len(conv), "max_conversion_rate": rate, "plan_stopped_by": why,
        "kv_cache_GB_unconverted_model": round(n_layers * kv_layer / 1e9, 2),
        "kv_cache_GB_after_conversion": round(n_soft * kv_layer / 1e9, 2),
        "dsla_states_GB": round(len(conv) * state_layer / 1e9, 3),
        "prefill_ms_all_layers": round(ms_prefill, 2),
        "prefill_ms_dsla_layers": round(ms_prefill_dsla, 2), "prefill_ms_softmax_layers": round(ms_prefill_soft, 2),
        "prefill_ms_if_no_layer_converted": round(ms_prefill_soft / max(n_soft, 1) * n_layers, 2),
        "softmax_prefill_TFLOPs_causal": round(n_soft * B * H * 2.0 * T * T * d * 2 / 2 / (ms_prefill_soft * 1e-3) / 1e12, 1) if soft else None,
        "decode_ms_per_token_all_layers": round(ms_decode, 3),
        "decode_ms_one_softmax_layer_full_cache": round(ms_decode_soft_layer, 4),
        "decode_ms_one_dsla_layer": round(ms_decode_dsla_layer, 4),
        "decode_ms_per_token_if_no_layer_converted": round(ms_decode_soft_layer * n_layers, 3),
        "request_ms_prompt_plus_decode": round(ms_prefill + decode * ms_decode, 1),
    }))


def project(M: int, K: int, H: int, d: int):
    """The projections in front of one layer (dsla_project: q, k, v and two gate pre-activations, 5 H d columns) and
    the prefill that consumes them; one JSON line."""
    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd import binding
    from paper_2506_09316_amd.binding import DSLA_BF16

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    width = H * d
    x = torch.randn(M, K, device=dev, generator=gen).to(torch.bfloat16)
    W = (torch.randn(5 * width, K, device=dev, generator=gen) * K ** -0.5).to(torch.bfloat16)
    outs = [torch.empty(1, M, H, d, device=dev, dtype=torch.bfloat16) for _ in range(5)]
    desc = dsla.make_desc(1, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, gamma=0.5, chunk=64, gate_mode=1, tau=16.0,
                          zero_init=True)
    S1, S2 = torch.empty(1, H, d, d, device=dev), torch.empty(1, H, d, d, device=dev)
    o = torch.empty_like(outs[2])
    nws = dsla.dsla_prefill_workspace_bytes(desc, M)
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device=dev)

    def step():
        dsla.dsla_project(x, W, outs)
        dsla.dsla_prefill(desc, M, outs[0], outs[1], outs[2], outs[3], outs[4], S1, S2, o, ws if nws else None)

    for _ in range(5):
        step()
    torch.cuda.synchronize()
    binding.profile_enable(True, 4096)
    for _ in range(20):
        step()
    res = binding.profile_collect()
    binding.profile_enable(False, 0)
    ms = {n: res[n][0] / res[n][1] for n in res if res[n][1]}
    flops = 2.0 * M * K * 5 * width
    print(json.dumps({"workload": f"projections of one layer: x [{M} x {K}] bf16 -> q, k, v, z1, z2 [{M} x {width}] each, then the "
                                  f"prefill with gate pre-activations (T = {M}, H = {H}, d = {d})",
                      "project_ms": round(ms["project"], 4), "project_TFLOPs": round(flops / (ms["project"] * 1e-3) / 1e12, 1),
                      "project_frac_of_bf16_mfma_peak": round(flops / (ms["project"] * 1e-3) / 1e12 / 2500.0, 4),
                      "prefill_kernels_ms": {n: round(v, 4) for n, v in ms.items() if n.startswith("prefill")}}))


def multi_state(N: int, Hkv: int, B: int, T: int, H: int, d: int):
    """dsla_decode_multi at the batched-decode shape and dsla_prefill_multi at the long-prompt shape for N states and
    H_kv key/value heads; one JSON line."""
    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd import binding
    from paper_2506_09316_amd.binding import DSLA_BF16

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    rnd = lambda *shape: (torch.randn(*shape, device=dev, generator=gen) * d ** -0.5).to(torch.bfloat16)

    def gates(*shape):
        z = torch.randn(*shape, device=dev, generator=gen) + 2.0
        return (-torch.nn.functional.softplus(-z) / 16.0).to(torch.bfloat16)

    w = [1.0 / N] * N
    # ---- decode: B = 64 sequences, rotating over several state sets so that the last-level cache cannot hold them
    Bd, NSETS = 64, max(2, 8 // N)
    desc = dsla.make_desc(Bd, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16)
    sets = [[torch.randn(Bd, H, d, d, device=dev, generator=gen) * 0.05 for _ in range(N)] for _ in range(NSETS)]
    q, k, v = rnd(Bd, H, d), rnd(Bd, Hkv, d), rnd(Bd, Hkv, d)
    ga = [gates(Bd, H, d) for _ in range(N)]
    o = torch.empty_like(q)
    multis = [dsla.make_multi(ga, s, w, H_kv=Hkv) for s in sets]
    for i in range(8):
        dsla.dsla_decode_multi(desc, multis[i % NSETS], q, k, v, o)
    torch.cuda.synchronize()
    binding.profile_enable(True, 4096)
    for i in range(64):
        dsla.dsla_decode_multi(desc, multis[i % NSETS], q, k, v, o)
    res = binding.profile_collect()
    us_dec = 1e3 * res["decode_multi"][0] / res["decode_multi"][1]
    dec_bytes = Bd * H * N * d * d * 4 * 2
    del sets, multis
    # ---- prefill: one long prompt
    pdesc = dsla.make_desc(B, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, chunk=64, zero_init=True)
    pq, pk, pv = rnd(B, T, H, d), rnd(B, T, Hkv, d), rnd(B, T, Hkv, d)
    pga = [gates(B, T, H, d) for _ in range(N)]
    S = [torch.empty(B, H, d, d, device=dev) for _ in range(N)]
    po = torch.empty_like(pq)
    pm = dsla.make_multi(pga, S, w, H_kv=Hkv)
    ws = torch.empty(max(dsla.dsla_prefill_multi_workspace_bytes(pdesc, pm, T), 256), dtype=torch.uint8, device=dev)
    for _ in range(5):
        dsla.dsla_prefill_multi(pdesc, pm, T, pq, pk, pv, po, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        dsla.dsla_prefill_multi(pdesc, pm, T, pq, pk, pv, po, ws)
    e1.record()
    torch.cuda.synchronize()
    binding.profile_enable(False, 0)
    ms_pre = e0.elapsed_time(e1) / 20
    print(json.dumps({"workload": f"N = {N} states, H = {H} query heads, H_kv = {Hkv}, d = {d}, bf16 io, fp32 states",
                      "decode_multi_us_B64": round(us_dec, 2), "decode_multi_GBps": round(dec_bytes / us_dec / 1e3, 1),
                      "decode_multi_frac_of_8TBps": round(dec_bytes / us_dec / 1e3 / 8000, 4),
                      "prefill_multi_ms": round(ms_pre, 4), "prefill_multi_tokens_per_s": round(B * T / (ms_pre * 1e-3), 1),
                      "prefill_shape": f"B={B} T={T}"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--attention-decode", action="store_true",
                    help="time the decode step of an unconverted softmax layer against the DSLA decode step instead")
    ap.add_argument("--attention-prefill", action="store_true",
                    help="time the causal softmax prefill of one unconverted layer instead")
    ap.add_argument("--entropy", action="store_true", help="time the attention-entropy kernel on one layer's keys instead")
    ap.add_argument("--packed", choices=sorted(MIXES), help="time one packed mixed-length prefill batch instead")
    ap.add_argument("--hybrid", action="store_true",
                    help="the whole hybrid configuration: --layers attention layers (default 32), the conversion logic "
                         "picks the DSLA ones, prompt and decode through every layer")
    ap.add_argument("--project", action="store_true", help="time the projection GEMM of one layer and the prefill behind it")
    ap.add_argument("--K", type=int, default=4096, help="--project: model width")
    ap.add_argument("--multi", type=int, default=0, metavar="N", help="time the N-state decode and prefill calls")
    ap.add_argument("--Hkv", type=int, default=0, help="--multi: key/value heads (default: H)")
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--B", type=int, default=8)
    ap.add_argument("--T", type=int, default=8192)
    ap.add_argument("--H", type=int, default=32)
    ap.add_argument("--d", type=int, default=128)
    ap.add_argument("--decode", type=int, default=128)
    ap.add_argument("--repeat", type=int, default=5, help="timed repetitions of the prefill of all layers")
    a = ap.parse_args()
    if a.project:
        return project(16384 if a.T == 8192 else a.T, a.K, a.H, a.d)
    if a.multi:
        return multi_state(a.multi, a.Hkv or a.H, 1 if a.B == 8 else a.B, 16384 if a.T == 8192 else a.T, a.H, a.d)
    if a.hybrid:
        return hybrid(a.layers or 32, a.B, a.T, a.H, a.d, a.decode)
    a.layers = a.layers or 16
    if a.packed:
        return packed(a.packed, a.H, a.d)
    if a.entropy:
        return entropy(a.B, a.T, a.H, a.d)
    if a.attention_decode:
        return attention_decode(a.B, a.T, a.H, a.d)
    if a.attention_prefill:
        return attention_prefill(a.B, a.T, a.H, a.d)

    import torch
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd.binding import DSLA_BF16

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250609)
    L, B, T, H, d = a.layers, a.B, a.T, a.H, a.d

    def rnd(*shape):
        return (torch.randn(*shape, device=dev, generator=gen) * d ** -0.5).to(torch.bfloat16)

    def gates(*shape):   # log alpha = -softplus(-z) / 16, z ~ N(2, 1)
        z = torch.randn(*shape, device=dev, generator=gen) + 2.0
        return (-torch.nn.functional.softplus(-z) / 16.0).to(torch.bfloat16)

    q, k, v, g1, g2 = rnd(B, T, H, d), rnd(B, T, H, d), rnd(B, T, H, d), gates(B, T, H, d), gates(B, T, H, d)
    o = torch.empty_like(v)
    gammas = torch.rand(L, generator=torch.Generator().manual_seed(7)) * 0.6 + 0.2
    descs = [dsla.make_desc(B, H, d, d, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, gamma=float(gammas[l]), chunk=64)
             for l in range(L)]
    S = [(torch.empty(B, H, d, d, device=dev), torch.empty(B, H, d, d, device=dev)) for _ in range(L)]
    nws = dsla.dsla_prefill_workspace_bytes(descs[0], T)
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device=dev)

    def prefill_all():
        for l in range(L):
            dsla.dsla_state_init(descs[l], *S[l])
            dsla.dsla_prefill(descs[l], T, q, k, v, g1, g2, S[l][0], S[l][1], o, ws)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    for _ in range(2):
        prefill_all()
    ms_prefill = timed(prefill_all, a.repeat)

    # decode: one token per sequence and layer; the inputs of a step live in fixed buffers (a real stack would
    # write its projections there), so one captured step serves every token
    dq, dk, dv, dg1, dg2 = rnd(L, B, H, d), rnd(L, B, H, d), rnd(L, B, H, d), gates(L, B, H, d), gates(L, B, H, d)
    do = torch.empty_like(dv)

    def decode_step():
        for l in range(L):
            dsla.dsla_decode(descs[l], dq[l], dk[l], dv[l], dg1[l], dg2[l], S[l][0], S[l][1], do[l])

    for _ in range(3):
        decode_step()
    ms_eager = timed(decode_step, a.decode)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        decode_step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        decode_step()
    graph.replay()
    ms_graph = timed(graph.replay, a.decode)
    assert bool(torch.isfinite(do.float()).all()) and bool(torch.isfinite(o.float()).all())

    # the other half of the hybrid stack at decode time: L softmax-attention layers, each over its own key/value
    # cache of T positions (the DSLA layers need no cache: that is the memory the conversion frees)
    caches = [(rnd(B, T, H, d), rnd(B, T, H, d)) for _ in range(L)]
    aq, ao = rnd(L, B, H, d), torch.empty(L, B, H, d, dtype=torch.bfloat16, device=dev)
    aws = torch.empty(max(dsla.dsla_attention_decode_workspace_bytes(B, H, d, T), 16), dtype=torch.uint8, device=dev)

    def softmax_layers():
        for l in range(L):
            dsla.dsla_attention_decode(aq[l], caches[l][0], caches[l][1], ao[l], d ** -0.5, aws)

    def hybrid_step():
        for l in range(L):
            dsla.dsla_attention_decode(aq[l], caches[l][0], caches[l][1], ao[l], d ** -0.5, aws)
            dsla.dsla_decode(descs[l], dq[l], dk[l], dv[l], dg1[l], dg2[l], S[l][0], S[l][1], do[l])

    for _ in range(2):
        hybrid_step()
    ms_softmax = timed(softmax_layers, 10)
    ms_hybrid = timed(hybrid_step, 10)
    assert bool(torch.isfinite(ao.float()).all())
    cache_bytes = L * 2 * B * T * H * d * 2

    state_bytes = L * B * H * (2 * d * d * 4 * 2 + 6 * d * 2)
    print(json.dumps({
        "workload": f"DSLA share of a serving step: {L} layer instances, B={B} H={H} d={d}, prompt T={T}, "
                    f"{a.decode} decode steps, bf16 io, fp32 states, synthetic inputs",
        "prefill_ms_all_layers": round(ms_prefill, 3),
        "prefill_layer_tokens_per_s": round(L * B * T / (ms_prefill * 1e-3), 1),
        "decode_step_ms_all_layers_eager": round(ms_eager, 4),
        "decode_step_ms_all_layers_graph": round(ms_graph, 4),
        "decode_layer_tokens_per_s_graph": round(L * B / (ms_graph * 1e-3), 1),
        "decode_GBps_graph": round(state_bytes / (ms_graph * 1e-3) / 1e9, 1),
        "request_ms_prompt_plus_decode": round(ms_prefill + a.decode * ms_graph, 2),
        "softmax_layers_decode_step_ms": round(ms_softmax, 4),
        "softmax_layers_kv_cache_GB": round(cache_bytes / 1e9, 2),
        "hybrid_decode_step_ms_softmax_plus_dsla_layers": round(ms_hybrid, 4),
        "attention_time_of_decode_unconverted_over_half_converted": round(2 * ms_softmax / ms_hybrid, 2),
    }))


if __name__ == "__main__":
    main()
