"""GPU parity of dsla_attention_entropy (the sensitivity signal of Section 4.3) and dsla_attention_decode (the
decode step of an unconverted softmax layer) against the fp64 oracle, element by element.  The arithmetic is fp32 on exact inputs (bf16 or fp32 values), so one tolerance holds for both
storage types: 1e-4 of the largest entropy in the tensor, plus special cases with known values."""
import math

import numpy as np
import pytest

import paper_2506_09316_amd as dsla
from oracle import attention as ent
import workloads as wl
from tests.util import max_rel_err, to_gpu

pytestmark = pytest.mark.gpu


def run(q_last, k, scale, io):
    import torch
    B, T, H, d = k.shape
    qg, kg = to_gpu(q_last, io), to_gpu(k, io)
    out = torch.full((B, H), float("nan"), device="cuda", dtype=torch.float32)
    n = dsla.dsla_attention_entropy_workspace_bytes(B, H, d, T)
    ws = torch.empty(n, dtype=torch.uint8, device="cuda") if n else None
    dsla.dsla_attention_entropy(qg, kg, out, scale, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), n


def inputs(seed, B, T, H, d, io, spread=1.0):
    x = wl.layer_inputs(seed, B, T + 1, H, d, d, io_dtype=io, gate_dtype="f32", qk_scale=1.0)
    k = x["k"][:, :T]
    q_last = x["q"][:, T] * np.float32(spread)
    if io == "bf16":
        q_last = wl.round_to_bf16(q_last)
    return q_last, k


@pytest.mark.parametrize("io,B,T,H,d", [("bf16", 2, 1000, 3, 128), ("bf16", 1, 4097, 2, 64), ("f32", 2, 700, 2, 128),
                                        ("f32", 1, 333, 4, 64), ("bf16", 3, 1, 2, 128), ("bf16", 1, 17, 1, 128),
                                        ("bf16", 70, 300, 8, 128)])
def test_entropy_against_oracle(io, B, T, H, d):
    q_last, k = inputs(7 + T, B, T, H, d, io)
    got, nws = run(q_last, k, d ** -0.5, io)
    ref = ent.attention_entropy(q_last, k, d ** -0.5)
    print(f"  B={B} T={T} H={H} d={d} {io}: workspace {nws} B, entropy range {ref.min():.4f} .. {ref.max():.4f}, "
          f"max err {np.max(np.abs(got - ref)):.2e}", flush=True)
    assert np.all(np.isfinite(got))
    if T == 1:
        assert np.all(np.abs(got) < 1e-6)
    else:
        assert max_rel_err(got, ref) < 1e-4


def test_entropy_peaked_and_flat_rows():
    """Sharp attention (large |q|: entropy far below log T, a few keys carry the row) and flat attention (q = 0:
    exactly log T), with the keys split over several workgroups."""
    B, T, H, d = 1, 6000, 2, 128
    q_last, k = inputs(11, B, T, H, d, "bf16", spread=6.0)
    got, nws = run(q_last, k, d ** -0.5, "bf16")
    assert nws > 0
    ref = ent.attention_entropy(q_last, k, d ** -0.5)
    assert ref.max() < 0.7 * math.log(T)
    assert np.max(np.abs(got - ref)) < 1e-4 * math.log(T)
    got, _ = run(np.zeros_like(q_last), k, 1.0, "bf16")
    assert np.max(np.abs(got - math.log(T))) < 1e-5 * math.log(T)


def test_entropy_full_size_sampled_heads():
    """The shape of the hybrid serving configuration (B = 8, H = 32, d = 128, T = 8192), all 256 rows computed,
    16 of them checked against the oracle."""
    B, T, H, d = 8, 8192, 32, 128
    rng = np.random.default_rng(13)
    k = wl.round_to_bf16(rng.standard_normal((B, T, H, d), dtype=np.float32))
    q_last = wl.round_to_bf16(rng.standard_normal((B, H, d), dtype=np.float32) * np.float32(1.5))
    got, nws = run(q_last, k, d ** -0.5, "bf16")
    assert np.all(np.isfinite(got))
    for b, h in [(b, (5 * b + j) % H) for b in range(B) for j in (0, 17)]:
        ref = ent.attention_entropy(q_last[b:b + 1, h:h + 1], k[b:b + 1, :, h:h + 1], d ** -0.5)[0, 0]
        assert abs(got[b, h] - ref) < 1e-4 * math.log(T), (b, h, got[b, h], ref)


# ---------------------------------------------------------------- single-query attention over a cache
def run_decode(q, k, v, scale, io):
    import torch
    B, T, H, d = k.shape
    qg, kg, vg = to_gpu(q, io), to_gpu(k, io), to_gpu(v, io)
    o = torch.full_like(qg, float("nan"))
    n = dsla.dsla_attention_decode_workspace_bytes(B, H, d, T)
    ws = torch.empty(n, dtype=torch.uint8, device="cuda") if n else None
    dsla.dsla_attention_decode(qg, kg, vg, o, scale, ws)
    torch.cuda.synchronize()
    return o.float().cpu().numpy(), n


@pytest.mark.parametrize("io,B,T,H,d,spread", [("bf16", 2, 1000, 3, 128, 1.0), ("bf16", 1, 4097, 2, 64, 1.0),
                                               ("f32", 2, 700, 2, 128, 1.0), ("f32", 1, 333, 4, 64, 3.0),
                                               ("bf16", 3, 1, 2, 128, 1.0), ("bf16", 1, 17, 1, 128, 5.0),
                                               ("bf16", 70, 300, 8, 128, 2.0), ("bf16", 1, 6000, 2, 128, 6.0)])
def test_attention_decode_against_oracle(io, B, T, H, d, spread):
    """Tolerances as for the DSLA layer (max |x - ref| / max |ref| over the tensor): fp32 1e-4; bf16 2e-2.  With
    bf16 the arithmetic is fp32 on exact inputs and the only rounding is that of the output (half a bf16 ulp, at
    most 2^-8 of the element), so the error is also held to 2^-8 plus a little."""
    q, k = inputs(21 + T, B, T, H, d, io, spread=spread)
    v = wl.layer_inputs(77 + T, B, T, H, d, d, io_dtype=io, gate_dtype="f32")["v"]
    got, nws = run_decode(q, k, v, d ** -0.5, io)
    ref = ent.attention_decode(q, k, v, d ** -0.5)
    err = max_rel_err(got, ref)
    print(f"  B={B} T={T} H={H} d={d} {io} spread={spread}: workspace {nws} B, max rel err {err:.2e}", flush=True)
    assert np.all(np.isfinite(got))
    assert err < (1e-4 if io == "f32" else 2e-2)
    if io == "bf16":
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.max(np.abs(ref)))


def test_attention_decode_full_size_sampled_heads():
    """B = 8, H = 32, d = 128, T = 8192 (the serving configuration's cache of one layer), 16 rows checked."""
    B, T, H, d = 8, 8192, 32, 128
    rng = np.random.default_rng(15)
    k = wl.round_to_bf16(rng.standard_normal((B, T, H, d), dtype=np.float32))
    v = wl.round_to_bf16(rng.standard_normal((B, T, H, d), dtype=np.float32))
    q = wl.round_to_bf16(rng.standard_normal((B, H, d), dtype=np.float32) * np.float32(2.0))
    got, _ = run_decode(q, k, v, d ** -0.5, "bf16")
    assert np.all(np.isfinite(got))
    for b, h in [(b, (7 * b + j) % H) for b in range(B) for j in (1, 20)]:
        ref = ent.attention_decode(q[b:b + 1, h:h + 1], k[b:b + 1, :, h:h + 1], v[b:b + 1, :, h:h + 1], d ** -0.5)[0, 0]
        assert np.all(np.abs(got[b, h] - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.max(np.abs(ref))), (b, h)


def test_attention_decode_mixed_context_lengths():
    """Requests of one batch at different context lengths in a cache of T positions each: only the filled positions
    count (the rest of the cache holds NaN here), also where a whole key range of the split lies past the end."""
    import torch
    B, T, H, d = 5, 3000, 2, 128
    lens = [3000, 1, 700, 1501, 37]
    q, k = inputs(31, B, T, H, d, "bf16", spread=2.0)
    v = wl.layer_inputs(33, B, T, H, d, d, io_dtype="bf16", gate_dtype="f32")["v"]
    kg, vg = to_gpu(k, "bf16"), to_gpu(v, "bf16")
    for b, L in enumerate(lens):
        kg[b, L:] = float("nan")
        vg[b, L:] = float("nan")
    qg = to_gpu(q, "bf16")
    o = torch.full_like(qg, float("nan"))
    n = dsla.dsla_attention_decode_workspace_bytes(B, H, d, T)
    assert n > 0
    ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    dsla.dsla_attention_decode(qg, kg, vg, o, d ** -0.5, ws, seq_lens=torch.tensor(lens, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    got = o.float().cpu().numpy()
    assert np.all(np.isfinite(got))
    for b, L in enumerate(lens):
        ref = ent.attention_decode(q[b:b + 1], k[b:b + 1, :L], v[b:b + 1, :L], d ** -0.5)[0]
        assert np.all(np.abs(got[b] - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.max(np.abs(ref))), (b, L)


# ---------------------------------------------------------------- causal attention over a prompt
def _run_attention_prefill(x, scale):
    import torch
    t = {n: to_gpu(x[n], "bf16") for n in ("q", "k", "v")}
    o = torch.full_like(t["v"], float("nan"))
    dsla.dsla_attention_prefill(t["q"], t["k"], t["v"], o, scale)
    torch.cuda.synchronize()
    return o.float().cpu().numpy()


@pytest.mark.parametrize("B,T,H,d,spread", [(2, 300, 3, 128, 1.0), (1, 129, 2, 64, 1.0), (1, 1, 2, 128, 1.0), (2, 31, 1, 64, 1.0),
                                            (1, 1000, 2, 128, 4.0), (3, 128, 2, 128, 1.0), (1, 2500, 1, 64, 2.0),
                                            (1, 65, 1, 128, 1.0), (2, 64, 2, 64, 1.0), (1, 193, 1, 128, 8.0)])
def test_attention_prefill_against_oracle(B, T, H, d, spread):
    """Every query position of a prompt against the definition (full score matrix, fp64): lengths on and off the
    boundaries of the 128-query and 64-key blocks, peaked and flat attention rows (the peaked ones raise the reference
    maximum of the kernel often, the flat ones once).  bf16 operands: the scores carry
    the rounding of scale * q to bf16 and the probabilities that of bf16, so the tolerance is the bf16 one of the
    DSLA path (2e-2 of the largest output)."""
    x = wl.layer_inputs(600 + T, B, T, H, d, d, io_dtype="bf16", gate_dtype="f32", qk_scale=1.0)
    x["q"] = wl.round_to_bf16(x["q"] * np.float32(spread))
    scale = d ** -0.5
    got = _run_attention_prefill(x, scale)
    ref = ent.attention_prefill(x["q"], x["k"], x["v"], scale)
    assert np.all(np.isfinite(got))
    err = max_rel_err(got, ref)
    print(f"    attention prefill B={B} T={T} H={H} d={d}: max rel err {err:.3e}", flush=True)
    assert err <= 2e-2
    np.testing.assert_allclose(got[:, 0], x["v"][:, 0], rtol=2 ** -7, atol=1e-6)   # the first position sees itself only


def test_attention_prefill_last_row_equals_attention_decode_and_full_size_sample():
    """B = 2, H = 8, T = 4096 at head size 128: sampled heads against the oracle, and the last query of every head
    against the single-query kernel on the same keys and values."""
    import torch
    B, T, H, d = 2, 4096, 8, 128
    x = wl.layer_inputs(650, B, T, H, d, d, io_dtype="bf16", gate_dtype="f32", qk_scale=1.0)
    scale = d ** -0.5
    got = _run_attention_prefill(x, scale)
    for b, h in ((0, 0), (1, 5)):
        xs = {n: x[n][b:b + 1, :, h:h + 1] for n in ("q", "k", "v")}
        ref = ent.attention_prefill(xs["q"], xs["k"], xs["v"], scale)
        err = max_rel_err(got[b:b + 1, :, h:h + 1], ref)
        print(f"    (b={b}, h={h}): max rel err {err:.3e}", flush=True)
        assert err <= 2e-2
    t = {n: to_gpu(x[n], "bf16") for n in ("q", "k", "v")}
    o1 = torch.empty(B, H, d, device="cuda", dtype=torch.bfloat16)
    n = dsla.dsla_attention_decode_workspace_bytes(B, H, d, T)
    ws = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")
    dsla.dsla_attention_decode(t["q"][:, T - 1].contiguous(), t["k"], t["v"], o1, scale, ws if n else None)
    torch.cuda.synchronize()
    assert max_rel_err(got[:, T - 1], o1.float().cpu().numpy()) <= 2e-2


def test_attention_prefill_argument_checks():
    import torch
    z = torch.zeros(1, 8, 2, 64, device="cuda")
    with pytest.raises(dsla.DslaError) as e:      # fp32 storage is not built for this call
        dsla.dsla_attention_prefill(z, z, z, z.clone(), 1.0)
    assert e.value.status == 3


def test_hybrid_stack_slice_against_oracles():
    """The hybrid configuration in miniature, at the real prompt length: 6 attention layers at B = 2, H = 32, d = 128,
    T = 8192; the library's conversion logic (entropy -> ranking -> plan capped by the prompt-length table) picks the
    layers that run as DSLA layers; every layer prefills the prompt and decodes 4 tokens (DSLA: prefill + decode
    step; softmax: causal attention + single-query attention over the growing cache).  One sampled (batch, head) pair
    per layer is held to the oracle of that layer's form."""
    import torch
    from oracle import dsla_oracle as orc
    B, T, H, d, L, steps = 2, 8192, 32, 128, 6, 4
    scale = d ** -0.5
    x = wl.layer_inputs(900, B, T + steps, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=1.0)
    t = {n: to_gpu(x[n], "bf16") for n in x}
    # sensitivities from the entropy kernel on per-layer scaled final queries (peaked .. flat)
    spreads = [6.0, 0.5, 3.0, 0.1, 9.0, 1.5]
    ent_out = torch.empty(B, H, device="cuda", dtype=torch.float32)
    n = dsla.dsla_attention_entropy_workspace_bytes(B, H, d, T)
    ews = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")
    sens = []
    for l in range(L):
        ql = wl.round_to_bf16(x["q"][:, T - 1] * np.float32(spreads[l]))
        dsla.dsla_attention_entropy(to_gpu(ql, "bf16"), t["k"][:, :T].contiguous(), ent_out, scale, ews if n else None)
        sens.append(float(ent_out.mean().item()))
    order = dsla.dsla_rank_layers(sens)
    assert order == sorted(range(L), key=lambda l: -spreads[l])      # the most peaked layer is the least sensitive
    kv = dsla.dsla_kv_cache_bytes(1, B, T + steps, H, d, 2)
    conv, _, why = dsla.dsla_conversion_plan(order, L * kv, 0, kv, B * H * 2 * d * d * 4, dsla.dsla_max_conversion_rate(T))
    assert len(conv) == 3 and why == "quality limit"                  # 50 % of 6 layers at a prompt of 8192 tokens
    qp, kp, vp = (t[n][:, :T].contiguous() for n in ("q", "k", "v"))
    g1p, g2p = t["g1"][:, :T].contiguous(), t["g2"][:, :T].contiguous()
    for l in range(L):
        b, h = l % B, (5 * l + 3) % H
        xs = {n: x[n][b:b + 1, :, h:h + 1] for n in x}
        o = torch.full_like(vp, float("nan"))
        if l in conv:
            gamma = 0.2 + 0.1 * l
            desc = dsla.make_desc(B, H, d, d, io_dtype=1, gate_dtype=1, gamma=gamma, scale=scale, chunk=64, zero_init=True)
            S1, S2 = torch.empty(B, H, d, d, device="cuda"), torch.empty(B, H, d, d, device="cuda")
            nb = dsla.dsla_prefill_workspace_bytes(desc, T)
            ws = torch.empty(max(nb, 1), dtype=torch.uint8, device="cuda")
            dsla.dsla_prefill(desc, T, qp, kp, vp, g1p, g2p, S1, S2, o, ws if nb else None)
            od = torch.empty(steps, B, H, d, device="cuda", dtype=torch.bfloat16)
            for s in range(steps):
                dsla.dsla_decode(desc, *(t[n][:, T + s].contiguous() for n in ("q", "k", "v", "g1", "g2")), S1, S2, od[s])
            torch.cuda.synchronize()
            ro, _, _ = orc.recurrent(xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], gamma, scale)
            got = np.concatenate([o[b, :, h].float().cpu().numpy(), od[:, b, h].float().cpu().numpy()])
        else:
            dsla.dsla_attention_prefill(qp, kp, vp, o, scale)
            nb = dsla.dsla_attention_decode_workspace_bytes(B, H, d, T + steps)
            ws = torch.empty(max(nb, 1), dtype=torch.uint8, device="cuda")
            od = torch.empty(steps, B, H, d, device="cuda", dtype=torch.bfloat16)
            for s in range(steps):
                lens = torch.full((B,), T + s + 1, dtype=torch.int32, device="cuda")
                dsla.dsla_attention_decode(t["q"][:, T + s].contiguous(), t["k"], t["v"], od[s], scale, ws if nb else None, seq_lens=lens)
            torch.cuda.synchronize()
            ro = ent.attention_prefill(xs["q"], xs["k"], xs["v"], scale)     # causal over prompt + decode tokens
            got = np.concatenate([o[b, :, h].float().cpu().numpy(), od[:, b, h].float().cpu().numpy()])
        err = max_rel_err(got, ro[0, :, 0])
        print(f"    layer {l} ({'DSLA' if l in conv else 'softmax'}), pair (b={b}, h={h}): max rel err {err:.3e}", flush=True)
        assert np.all(np.isfinite(got)) and err <= 2e-2
