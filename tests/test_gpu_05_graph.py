"""The library under HIP graph capture: it allocates nothing, never synchronises and enqueues only kernels on the
caller's stream, so a serving loop can capture its launch-bound part (one decode step of every layer, or a prefill)
once and replay it.  Every replay is compared with the same work issued eagerly."""
import numpy as np
import pytest

import paper_2506_09316_amd as dsla
import workloads as wl
from tests.util import code, to_gpu

pytestmark = pytest.mark.gpu


def _decode_inputs(seed, layers, B, H, d):
    x = wl.layer_inputs(seed, layers, B, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=d ** -0.5)
    return [{n: to_gpu(x[n][l], "bf16") for n in x} for l in range(layers)]


def test_decode_step_of_several_layers_replayed():
    import torch
    layers, B, H, d, replays = 4, 6, 8, 128, 4
    xs = _decode_inputs(5, layers, B, H, d)
    descs = [dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.2 + 0.15 * l)
             for l in range(layers)]
    S0 = [tuple(torch.from_numpy(a).cuda() for a in wl.initial_states(100 + l, B, H, d, d, amplitude=0.2))
          for l in range(layers)]

    def fresh():
        return [(a.clone(), b.clone()) for a, b in S0], [torch.full_like(x["v"], float("nan")) for x in xs]

    def step(S, o):
        for l in range(layers):
            x = xs[l]
            dsla.dsla_decode(descs[l], x["q"], x["k"], x["v"], x["g1"], x["g2"], S[l][0], S[l][1], o[l])

    # eager: the outputs of every step
    S_e, o_e = fresh()
    want = []
    for _ in range(replays):
        step(S_e, o_e)
        torch.cuda.synchronize()
        want.append([t.clone() for t in o_e])

    # captured once, replayed with eager work and synchronisation between the replays
    S_g, o_g = fresh()
    warm_S, warm_o = fresh()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):      # warm-up outside the capture (loads the code objects)
        step(warm_S, warm_o)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(S_g, o_g)
    # the capture itself runs nothing
    assert all(torch.equal(a, b) for (a, _), (b, _) in zip(S_g, S0))
    for r in range(replays):
        graph.replay()
        torch.cuda.synchronize()
        for l in range(layers):
            assert torch.equal(o_g[l], want[r][l]), f"replay {r}, layer {l}"
        step(warm_S, warm_o)           # unrelated eager work between replays
        torch.cuda.synchronize()
    for l in range(layers):
        assert torch.equal(S_g[l][0], S_e[l][0]) and torch.equal(S_g[l][1], S_e[l][1])


def test_prefill_with_segments_replayed():
    """A captured prefill (three kernels and a workspace) replayed on new input values in the same buffers."""
    import torch
    B, T, H, d = 1, 1000, 4, 128
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.4, chunk=64, segments=4)
    bufs = {n: torch.empty(B, T, H, d, dtype=torch.bfloat16, device="cuda") for n in ("q", "k", "v", "g1", "g2")}
    o = torch.empty(B, T, H, d, dtype=torch.bfloat16, device="cuda")
    S1 = torch.zeros(B, H, d, d, device="cuda")
    S2 = torch.zeros_like(S1)
    ws = torch.empty(dsla.dsla_prefill_workspace_bytes(desc, T), dtype=torch.uint8, device="cuda")

    def call(S1_, S2_, o_):
        dsla.dsla_state_init(desc, S1_, S2_)
        dsla.dsla_prefill(desc, T, bufs["q"], bufs["k"], bufs["v"], bufs["g1"], bufs["g2"], S1_, S2_, o_, ws)

    def load(seed):
        x = wl.layer_inputs(seed, B, T, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=d ** -0.5)
        for n in bufs:
            bufs[n].copy_(to_gpu(x[n], "bf16"))

    load(1)
    call(S1, S2, o)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(S1, S2, o)
    for seed in (2, 3, 2):
        load(seed)
        eS1, eS2, eo = torch.empty_like(S1), torch.empty_like(S2), torch.empty_like(o)
        call(eS1, eS2, eo)
        torch.cuda.synchronize()
        o.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, eo) and torch.equal(S1, eS1) and torch.equal(S2, eS2), f"seed {seed}"


def test_kernel_timing_leaves_results_alone_and_counts_every_launch():
    """dsla_profile_enable attaches a pair of events to every launch (the dispatches carry them).  A segmented
    prefill, decode steps and the two attention passes -- with one part per pair (no merge kernel) and with several --
    give bit-identical results with and without the timing, every launch is counted once, and every duration is
    positive and plausible."""
    import numpy as np
    import torch
    import workloads as wl
    import paper_2506_09316_amd as dsla
    from paper_2506_09316_amd import binding
    from tests.util import GpuLayer, slice_t, to_gpu

    B, T, H, d, steps = 1, 1024, 2, 128, 3
    x = wl.layer_inputs(505, B, T + steps, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=d ** -0.5)

    def layer_run():
        layer = GpuLayer(B, H, d, "bf16", "bf16", gamma=0.4, chunk=64, segments=4)
        outs = [layer.prefill(slice_t(x, 0, T))]
        for t in range(T, T + steps):
            outs.append(layer.decode(slice_t(x, t, t + 1)))
        return np.concatenate(outs, 1), layer.states()

    def attention_run(Ta):
        k = to_gpu(x["k"][:, :Ta], "bf16")
        v = to_gpu(x["v"][:, :Ta], "bf16")
        q = to_gpu(x["q"][:, Ta], "bf16")
        o = torch.full_like(q, float("nan"))
        e = torch.full((B, H), float("nan"), device="cuda", dtype=torch.float32)
        n = dsla.dsla_attention_decode_workspace_bytes(B, H, d, Ta)
        ws = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")
        dsla.dsla_attention_decode(q, k, v, o, d ** -0.5, ws if n else None)
        n = dsla.dsla_attention_entropy_workspace_bytes(B, H, d, Ta)
        ws2 = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")
        dsla.dsla_attention_entropy(q, k, e, d ** -0.5, ws2 if n else None)
        torch.cuda.synchronize()
        return o.float().cpu().numpy(), e.cpu().numpy()

    plain = (layer_run(), attention_run(17), attention_run(1000))
    binding.profile_enable(True, 64)
    try:
        timed = (layer_run(), attention_run(17), attention_run(1000))
        torch.cuda.synchronize()
        res = binding.profile_collect()
    finally:
        binding.profile_enable(False, 0)
    (o0, (a0, b0)), (o1, (a1, b1)) = plain[0], timed[0]
    assert np.array_equal(o0, o1) and np.array_equal(a0, a1) and np.array_equal(b0, b1)
    for p, t in zip(plain[1:], timed[1:]):
        assert np.array_equal(p[0], t[0]) and np.array_equal(p[1], t[1])
    print("  kernel timing:", {k: (round(ms * 1e3, 1), n) for k, (ms, n) in res.items() if n}, flush=True)
    expected = {"prefill_segment_state": 1, "prefill_segment_scan": 1, "prefill_chunk_loop": 1, "decode": steps,
                "attention_decode": 2, "attention_entropy": 2}
    for name, count in expected.items():
        ms, n = res[name]
        assert n == count, (name, n)
        assert 0.0 < ms / n < 5.0, (name, ms)      # microseconds to a few milliseconds per launch
