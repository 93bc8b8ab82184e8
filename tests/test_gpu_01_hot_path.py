"""GPU parity of the DSLA hot path: dsla_prefill, dsla_decode and dsla_state_init through the C ABI against the
CPU oracle, element by element.  The bf16 path that the benchmark times and the BASELINE configurations run first;
tolerances and norms are in tests/gpu_common.py."""
import numpy as np
import pytest

from oracle import dsla_oracle as orc
import workloads as wl
import paper_2506_09316_amd as dsla
from tests.gpu_common import TOL, check, run_prefill_case
from tests.util import GpuLayer, code, max_rel_err, slice_t, to_gpu

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------- carried states with several segments
@pytest.mark.parametrize("io,d,chunk", [("bf16", 128, 128), ("f32", 64, 64), ("bf16", 64, 32), ("f32", 128, 64)])
def test_carried_states_short_last_segment(io, d, chunk):
    """States carried into a call that is cut into segments whose last one is much shorter than the first
    (T = segment length + 1): the workgroup of the last segment finishes, and overwrites the caller's states, long
    before the workgroup of the first segment would be done; every segment must still start from the states as they
    were on entry.  Several (batch, head) pairs, dense and packed entry points."""
    import torch
    seg = 2 * chunk                               # tokens per segment the plans below arrive at
    T, B, H = seg + 1, 3, 4
    gd = "bf16" if io == "bf16" else "f32"
    run_prefill_case(B, T, H, d, io, gd, chunk=chunk, segments=2, gamma=0.6, seed=13, init=True, qk_scale=d ** -0.5)
    # the same through the packed entry point: sequences of seg + 1, 2 seg + 1 and 1 tokens in a pool of states
    lengths, slots, n_slots = [seg + 1, 2 * seg + 1, 1], [2, 0, 3], 4
    total = sum(lengths)
    x = wl.layer_inputs(14, 1, total, H, d, d, io_dtype=io, gate_dtype=gd, qk_scale=d ** -0.5)
    S1_0, S2_0 = wl.initial_states(15, n_slots, H, d, d, amplitude=2.0)
    desc = dsla.make_desc(len(lengths), H, d, d, io_dtype=code(io), gate_dtype=code(gd), gamma=0.6, chunk=chunk, segments=3)
    S1, S2 = (torch.from_numpy(a.copy()).cuda() for a in (S1_0, S2_0))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    t = {n: to_gpu(x[n][0], io if n in ("q", "k", "v") else gd) for n in x}
    o = torch.full_like(t["v"], float("nan"))
    nbytes = dsla.dsla_prefill_varlen_workspace_bytes(desc, total, max(lengths))
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")
    dsla.dsla_prefill_varlen(desc, total, max(lengths), torch.from_numpy(cu).cuda(),
                             torch.tensor(slots, dtype=torch.int32, device="cuda"), t["q"], t["k"], t["v"], t["g1"],
                             t["g2"], S1, S2, o, ws)
    torch.cuda.synchronize()
    o = o.float().cpu().numpy()
    for b, sl in enumerate(slots):
        r = slice(cu[b], cu[b + 1])
        ro, rS1, rS2 = orc.recurrent(x["q"][:, r], x["k"][:, r], x["v"][:, r], x["g1"][:, r], x["g2"][:, r], 0.6,
                                     S1=S1_0[sl:sl + 1], S2=S2_0[sl:sl + 1])
        check(f"packed o[seq {b}]", o[r][None], ro, TOL[io])
        check(f"packed S1[seq {b}]", S1[sl:sl + 1].cpu().numpy(), rS1, TOL[io])
        check(f"packed S2[seq {b}]", S2[sl:sl + 1].cpu().numpy(), rS2, TOL[io])

@pytest.mark.parametrize("io,d,B,H,T,chunk,init", [("bf16", 128, 4, 32, 1024, 0, False), ("bf16", 128, 3, 32, 1500, 64, True),
                                                   ("f32", 64, 2, 4, 512, 64, True), ("f32", 128, 1, 2, 700, 64, True),
                                                   ("bf16", 128, 2, 2, 1400, 128, False)])
def test_prefill_pre_pass_on_half_segments(io, d, B, H, T, chunk, init):
    """Plans of two segments that the library makes itself (no segment count given): the pre-pass, which would have a
    workgroup for at most half of the compute units, works on the two halves of the first segment, the scan combines
    them and the second segment of the chunk loop starts from slot 2.  The workspace size shows that the case is one
    of those (3 state slots and 2 decay vectors per (sequence, head)); the results are held to the oracle like any
    other."""
    gd = "bf16" if io == "bf16" else "f32"
    desc = dsla.make_desc(B, H, d, d, io_dtype=code(io), gate_dtype=code(gd), chunk=chunk)
    decay = 2 * B * H * 2 * d * 4
    assert dsla.dsla_prefill_workspace_bytes(desc, T) == 3 * B * H * 2 * d * d * 4 + (decay + 255) // 256 * 256
    run_prefill_case(B, T, H, d, io, gd, chunk=chunk, segments=0, gamma=0.35, seed=91, init=init, qk_scale=d ** -0.5)


@pytest.mark.parametrize("io,d,segments,T", [("bf16", 128, 1, 300), ("bf16", 128, 4, 1000), ("f32", 64, 1, 77),
                                             ("f32", 64, 3, 450)])
def test_prefill_zero_init_does_not_read_the_states(io, d, segments, T):
    """desc.zero_init: the states are zero by contract, the call only writes them (dsla_state_init folded in).
    The state tensors hold NaN on entry, so any read of them would show in the results."""
    B, H = 2, 3
    gd = "bf16" if io == "bf16" else "f32"
    x = wl.layer_inputs(61, B, T, H, d, d, io_dtype=io, gate_dtype=gd, qk_scale=d ** -0.5)
    layer = GpuLayer(B, H, d, io, gd, gamma=0.3, chunk=64, segments=segments, zero_init=True, init=False)
    o = layer.prefill(x)
    S1, S2 = layer.states()
    ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], x["g1"], x["g2"], 0.3)
    check("o", o, ro, TOL[io])
    check("S1", S1, rS1, TOL[io])
    check("S2", S2, rS2, TOL[io])


# ---------------------------------------------------------------- prefill, bf16


@pytest.mark.parametrize("d,chunk,segments,T,gd", [(128, 64, 1, 512, "bf16"), (128, 64, 3, 500, "f32"),
                                                   (128, 32, 2, 257, "bf16"), (64, 64, 2, 384, "bf16"),
                                                   (64, 32, 1, 100, "f32"), (128, 64, 0, 1024, "bf16")])
def test_prefill_bf16_shapes(d, chunk, segments, T, gd):
    run_prefill_case(2, T, 3, d, "bf16", gd, chunk=chunk, segments=segments, gamma=0.4, seed=21, init=True,
                     qk_scale=d ** -0.5)


@pytest.mark.parametrize("chunk,segments,T,tau,gate_mean", [(32, 8, 256, 16.0, 2.0), (32, 3, 200, 16.0, 2.0),
                                                            (64, 2, 1000, 16.0, 2.0), (64, 5, 1601, 16.0, 2.0),
                                                            (64, 2, 900, 1.0, -2.0), (128, 3, 2500, 4.0, 0.0)])
def test_prefill_segment_states_walked_backwards(chunk, segments, T, tau, gate_mean):
    """bf16 io and gates at d = 128: the state contribution of every segment but the last comes from the kernel that
    walks the segment backwards with suffix sums of the log-gates as exponents.  Segments of 1, 3, 16, 5 and 14 steps of
    32 tokens, a ragged last segment, carried-in states; weak gates and gates so strong (68 per 32 tokens) that the
    factors of the early tokens of a segment underflow to zero, as their true weights do."""
    run_prefill_case(2, T, 3, 128, "bf16", "bf16", chunk=chunk, segments=segments, gamma=0.55, tau=tau, seed=27, init=True,
                     gate_mean=gate_mean, qk_scale=128 ** -0.5)


@pytest.mark.parametrize("io,d,segments,T", [("bf16", 128, 2, 700), ("bf16", 128, 0, 4096), ("f32", 64, 3, 450)])
def test_prefill_chunk128(io, d, segments, T):
    run_prefill_case(1, T, 2, d, io, "f32" if io == "f32" else "bf16", chunk=128, segments=segments, gamma=0.45, seed=23,
                     init=True, qk_scale=d ** -0.5)


def test_prefill_bf16_strong_decay_tau1():
    run_prefill_case(1, 512, 4, 128, "bf16", "f32", chunk=64, segments=2, gamma=0.5, tau=1.0, seed=31,
                     qk_scale=128 ** -0.5)


def test_prefill_bf16_negative_blend_factors():
    """gamma > 1 makes the recency factor negative, a negative scale flips both: the sign travels in the packed
    bf16 Q~ operand (its magnitude in the exponent)."""
    run_prefill_case(1, 300, 2, 128, "bf16", "bf16", chunk=64, segments=2, gamma=1.3, scale=1.0, seed=41, init=True,
                     qk_scale=128 ** -0.5)
    run_prefill_case(1, 200, 2, 64, "bf16", "f32", chunk=32, segments=1, gamma=0.4, scale=-0.5, seed=43, init=True,
                     qk_scale=64 ** -0.5)
    run_prefill_case(1, 100, 2, 128, "bf16", "bf16", chunk=64, segments=1, gamma=0.0, scale=1.0, seed=45, init=True,
                     qk_scale=128 ** -0.5)


# ---------------------------------------------------------------- full-size configurations, sampled heads


def _full_size_check(cfg_name, heads=None, segments=0, chunk=None):
    """A BASELINE configuration at full size, in the launch configuration the benchmark times (automatic segment
    split); `heads` = the heads compared with the oracle (default: all of them)."""
    c = wl.CONFIGS[cfg_name]
    B, T, H, d = c["B"], c["T"], c["H"], c["dk"]
    chunk = chunk or c["chunk"]
    print(f"  {cfg_name}: B={B} T={T} H={H} d={d} chunk={chunk}", flush=True)
    x = wl.layer_inputs(c["seed"], B, T, H, d, d, io_dtype=c["io_dtype"], gate_dtype=c["gate_dtype"],
                        qk_scale=c["qk_scale"])
    layer = GpuLayer(B, H, d, c["io_dtype"], c["gate_dtype"], gamma=0.5, chunk=chunk, segments=segments)
    o = layer.prefill(x)
    S1, S2 = layer.states()
    assert np.all(np.isfinite(o))
    if heads is None:
        ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], x["g1"], x["g2"], 0.5)
        check("o", o, ro, 2e-2)
        check("S1", S1, rS1, 2e-2)
        check("S2", S2, rS2, 2e-2)
        return
    for h in heads:
        xs = {n: x[n][:, :, h:h + 1] for n in x}
        ro, rS1, rS2 = orc.recurrent(xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], 0.5)
        check(f"o[h={h}]", o[:, :, h:h + 1], ro, 2e-2)
        check(f"S1[h={h}]", S1[:, h:h + 1], rS1, 2e-2)
        check(f"S2[h={h}]", S2[:, h:h + 1], rS2, 2e-2)


def test_cfg2_full_size_all_heads():
    _full_size_check("cfg2")


def test_cfg3_16k_full_size_all_heads():
    """The workload bench.py times, every head and every token against the oracle."""
    _full_size_check("cfg3_16k")


def test_cfg3_16k_chunk128_all_heads():
    _full_size_check("cfg3_16k", chunk=128)


def test_cfg3_64k_full_size_all_heads():
    _full_size_check("cfg3_64k")


def test_cfg3_64k_chunk128_sampled_heads():
    _full_size_check("cfg3_64k", heads=(11, 29), chunk=128)


# ---------------------------------------------------------------- batched decode at full size (cfg4)


def test_cfg4_batched_decode_full_size_sampled_pairs():
    """B=64, H=32, d=128: states from a T=2048 prefill, then 256 fused decode steps on the full batch, in the
    launch configuration bench.py times.  The prefill tokens of sequence b are those of base sequence b % 4 (four
    seeded base sequences keep host generation small); decode inputs are distinct for all 64 sequences.  Sampled
    (batch, head) pairs are checked element by element against the oracle run over prefill + decode tokens."""
    import torch
    import paper_2506_09316_amd as dsla
    from tests.util import code, to_gpu
    c = wl.CONFIGS["cfg4"]
    B, T, H, d, steps, NB = c["B"], c["T"], c["H"], c["dk"], c["decode_steps"], 4
    base = wl.layer_inputs(c["seed"], NB, T, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=c["qk_scale"])
    dec = wl.layer_inputs(c["seed"] + 50, B, steps, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=c["qk_scale"])
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.5, chunk=c["chunk"])
    S1 = torch.empty(B, H, d, d, device="cuda")
    S2 = torch.empty_like(S1)
    dsla.dsla_state_init(desc, S1, S2)
    xg = {n: to_gpu(base[n], "bf16").repeat(B // NB, 1, 1, 1).contiguous() for n in base}  # sequence b <- base b % 4
    o = torch.empty_like(xg["v"])
    assert dsla.dsla_prefill_workspace_bytes(desc, T) == 0
    dsla.dsla_prefill(desc, T, xg["q"], xg["k"], xg["v"], xg["g1"], xg["g2"], S1, S2, o, None)
    torch.cuda.synchronize()
    pairs = ((0, 0), (5, 17), (34, 3), (63, 31), (22, 9))
    o_pre = {(b, h): o[b, :, h].float().cpu().numpy() for b, h in pairs}
    assert bool(torch.isfinite(o.float()).all())
    del xg, o
    dg = {n: to_gpu(dec[n], "bf16") for n in dec}   # [B, steps, H, d]
    outs = torch.empty(steps, B, H, d, device="cuda", dtype=torch.bfloat16)
    for t in range(steps):
        dsla.dsla_decode(desc, dg["q"][:, t].contiguous(), dg["k"][:, t].contiguous(), dg["v"][:, t].contiguous(),
                         dg["g1"][:, t].contiguous(), dg["g2"][:, t].contiguous(), S1, S2, outs[t])
    torch.cuda.synchronize()
    o_dec = outs.float().cpu().numpy()           # [steps, B, H, d]
    S1h, S2h = S1.cpu().numpy(), S2.cpu().numpy()
    assert np.all(np.isfinite(o_dec))
    for b, h in pairs:
        x = {n: np.concatenate([base[n][b % NB:b % NB + 1, :, h:h + 1], dec[n][b:b + 1, :, h:h + 1]], 1) for n in base}
        ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], x["g1"], x["g2"], 0.5)
        print(f"  pair (b={b}, h={h})", flush=True)
        check("o prefill", o_pre[(b, h)], ro[0, :T, 0], 2e-2)
        check("o decode", o_dec[:, b, h], ro[0, T:, 0], 2e-2)
        check("S1", S1h[b, h], rS1[0, 0], 2e-2)
        check("S2", S2h[b, h], rS2[0, 0], 2e-2)


def test_cfg5_layer_instances_slice():
    """The DSLA part of the hybrid serving step: several layer instances, each with its own blend coefficient and
    inputs, prefill T=8192 then 128 decode steps.  A slice is checked: 3 of the 16 layers, 2 of the 8 sequences,
    2 heads each, element by element against the oracle over prefill + decode tokens."""
    c = wl.CONFIGS["cfg5"]
    T, H, d, steps, B = c["T"], c["H"], c["dk"], c["decode_steps"], 2
    for layer_no in (0, 7, 15):
        seed = c["seed"] + 10 * layer_no
        gamma = float(np.random.default_rng(seed + 9).uniform(0.2, 0.8))
        print(f"  layer {layer_no}: gamma={gamma:.4f}", flush=True)
        x = wl.layer_inputs(seed, B, T + steps, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=c["qk_scale"])
        layer = GpuLayer(B, H, d, "bf16", "bf16", gamma=gamma, chunk=c["chunk"])
        outs = [layer.prefill(slice_t(x, 0, T))]
        for t in range(T, T + steps):
            outs.append(layer.decode(slice_t(x, t, t + 1)))
        o = np.concatenate(outs, 1)
        S1, S2 = layer.states()
        assert np.all(np.isfinite(o))
        for b, h in ((0, 3 + layer_no), (1, 20)):
            xs = {n: x[n][b:b + 1, :, h:h + 1] for n in x}
            ro, rS1, rS2 = orc.recurrent(xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], gamma)
            check(f"o prefill[b={b},h={h}]", o[b:b + 1, :T, h:h + 1], ro[:, :T], 2e-2)
            check(f"o decode[b={b},h={h}]", o[b:b + 1, T:, h:h + 1], ro[:, T:], 2e-2)
            check(f"S1[b={b},h={h}]", S1[b:b + 1, h:h + 1], rS1, 2e-2)
            check(f"S2[b={b},h={h}]", S2[b:b + 1, h:h + 1], rS2, 2e-2)


# ---------------------------------------------------------------- decode


@pytest.mark.parametrize("io,gd,d", [("f32", "f32", 64), ("bf16", "bf16", 128), ("bf16", "f32", 64), ("f32", "bf16", 128)])
def test_decode_steps(io, gd, d):
    B, H, steps = 3, 5, 6
    x = wl.layer_inputs(77, B, steps, H, d, d, io_dtype=io, gate_dtype=gd, tau=4.0)
    S10, S20 = wl.initial_states(78, B, H, d, d)
    gph = np.linspace(0.1, 0.9, H)
    layer = GpuLayer(B, H, d, io, gd, scale=0.5, gamma_per_head=gph)
    layer.set_states(S10, S20)
    s1, s2 = S10.astype(np.float64), S20.astype(np.float64)
    for t in range(steps):
        xt = slice_t(x, t, t + 1)
        o = layer.decode(xt)
        ro, s1, s2 = orc.recurrent(xt["q"], xt["k"], xt["v"], xt["g1"], xt["g2"], gph, 0.5, S1=s1, S2=s2)
        # o is rounded to the I/O dtype on the way out: one bf16 ulp is 2^-8 relative
        check(f"o[{t}]", o, ro, TOL[io])
    S1, S2 = layer.states()
    check("S1", S1, s1, 1e-5)
    check("S2", S2, s2, 1e-5)


# ---------------------------------------------------------------- prefill, fp32 (tight check of the algebra)


def test_prefill_cfg1_fp32():
    c = wl.CONFIGS["cfg1"]
    for gamma, tau in ((0.5, 16.0), (0.3, 16.0), (0.5, 1.0)):
        run_prefill_case(c["B"], c["T"], c["H"], c["dk"], "f32", "f32", chunk=c["chunk"], gamma=gamma, tau=tau,
                         seed=c["seed"])


@pytest.mark.parametrize("chunk,segments,T", [(64, 1, 256), (64, 2, 256), (64, 4, 256), (32, 1, 256), (32, 3, 224),
                                              (64, 1, 200), (64, 3, 333), (32, 2, 37), (64, 1, 1), (32, 1, 31),
                                              (64, 0, 2048)])
def test_prefill_fp32_shapes(chunk, segments, T):
    run_prefill_case(2, T, 3, 64, "f32", "f32", chunk=chunk, segments=segments, gamma=0.35, scale=0.7, seed=5,
                     init=True, gph=None)


def test_prefill_fp32_d128_chunk32_per_head_gamma():
    run_prefill_case(1, 150, 2, 128, "f32", "bf16", chunk=32, segments=2, seed=9, init=True, gph=np.array([0.2, 0.9]),
                     qk_scale=128 ** -0.5)


def test_prefill_fp32_d128_chunk64():
    run_prefill_case(1, 200, 2, 128, "f32", "f32", chunk=64, segments=2, gamma=0.6, seed=13, init=True,
                     qk_scale=128 ** -0.5)


@pytest.mark.parametrize("io,gd,d", [("f32", "f32", 64), ("bf16", "f32", 128), ("bf16", "bf16", 128), ("f32", "f32", 128)])
@pytest.mark.parametrize("chunk", [64, 128])
@pytest.mark.parametrize("gate_mean", [0.0, -2.0])
def test_prefill_plain_sigmoid_gates(io, gd, d, chunk, gate_mean):
    """tau = 1 (plain sigmoid) gates with pre-activations z ~ N(0, 1) and z ~ N(-2, 1): |log alpha| averages 0.8 and
    2.1 per token, 26 and 68 per 32 tokens, 52 and 136 per chunk of 64; the recency state then forgets within a few
    tokens.  The exponents are referred to the middle of each group of 32 tokens, so neither the chunk length nor the
    sequence length limits the decay; carried-in states, several segments, a ragged end."""
    run_prefill_case(2, 5 * chunk + 37, 2, d, io, gd, chunk=chunk, segments=2, gamma=0.5, tau=1.0, seed=17, init=True,
                     gate_mean=gate_mean, qk_scale=d ** -0.5)


def test_prefill_gates_of_any_strength_when_not_sustained():
    """Single tokens that all but close a gate (log alpha = -100 and -120, alpha = 4e-44 and 8e-53) among ordinary
    ones: the state is wiped at those tokens, and the sum over their group of 32 stays inside the domain because they
    are single; another group is filled with as much sustained decay as the domain allows (32 tokens of alpha = 0.0074)."""
    B, T, H, d = 1, 200, 2, 64
    x = wl.layer_inputs(71, B, T, H, d, d, io_dtype="f32", gate_dtype="f32", qk_scale=d ** -0.5)
    x["g1"][:, 40, :, ::3] = np.float32(-100.0)
    x["g2"][:, 41, :, 1::3] = np.float32(-120.0)
    x["g1"][:, 96:128, :, 5] = np.float32(-4.9)     # 32 tokens of alpha = 0.0074: 157 over the group
    from tests.gpu_common import GATE_DOMAIN, step_gate_sums
    assert 150.0 < step_gate_sums(x) < GATE_DOMAIN
    import torch
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    layer = GpuLayer(B, H, d, "f32", "f32", gamma=0.4, chunk=64, segments=2, status=status)
    o = layer.prefill(x)
    S1, S2 = layer.states()
    ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], x["g1"], x["g2"], 0.4)
    check("o", o, ro, 1e-4)
    check("S1", S1, rS1, 1e-4)
    check("S2", S2, rS2, 1e-4)
    assert int(status.item()) == 0


def test_prefill_reports_gates_outside_the_domain():
    """Sustained gates of 3e-4 (log alpha = -8 on every token: 256 over 32 tokens) are outside the domain: the kernels
    say so through the status word instead of returning silently; features that stay inside are still right."""
    import torch
    B, T, H, d = 1, 96, 1, 64
    x = wl.layer_inputs(73, B, T, H, d, d, io_dtype="f32", gate_dtype="f32", qk_scale=d ** -0.5)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    layer = GpuLayer(B, H, d, "f32", "f32", gamma=0.5, chunk=32, segments=1, status=status)
    layer.prefill(x)
    assert int(status.item()) == 0
    x["g2"][:, 32:64, :, 7] = np.float32(-8.0)
    layer.prefill(x)
    assert int(status.item()) == 1


def test_prefill_fp32_gamma_extremes():
    for gamma in (0.0, 1.0, 1.5):
        run_prefill_case(1, 130, 2, 64, "f32", "f32", chunk=64, segments=2, gamma=gamma, seed=11, init=True)


# ---------------------------------------------------------------- invariants on the GPU path


def test_continuation_prefill_prefill_decode():
    """prefill(T1) -> prefill(T2) -> n decode steps equals the oracle over T1 + T2 + n tokens."""
    B, H, d, T1, T2, n = 1, 4, 64, 100, 156, 16
    c = wl.CONFIGS["cfg1"]
    x = wl.layer_inputs(c["seed"] + 7, B, T1 + T2 + n, H, d, d, io_dtype="f32", gate_dtype="f32")
    layer = GpuLayer(B, H, d, "f32", "f32", gamma=0.5, chunk=64)
    outs = [layer.prefill(slice_t(x, 0, T1)), layer.prefill(slice_t(x, T1, T1 + T2))]
    for t in range(T1 + T2, T1 + T2 + n):
        outs.append(layer.decode(slice_t(x, t, t + 1)))
    o = np.concatenate(outs, 1)
    S1, S2 = layer.states()
    ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], x["g1"], x["g2"], 0.5)
    check("o", o, ro, 1e-4)
    check("S1", S1, rS1, 1e-4)
    check("S2", S2, rS2, 1e-4)


def test_chunk_and_segment_invariance_and_determinism():
    B, T, H, d = 1, 512, 2, 128
    x = wl.layer_inputs(41, B, T, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=d ** -0.5)
    outs = []
    for chunk, seg in ((64, 1), (64, 1), (64, 4), (32, 2), (128, 2)):
        layer = GpuLayer(B, H, d, "bf16", "bf16", chunk=chunk, segments=seg)
        outs.append((layer.prefill(x),) + layer.states())
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b), "same call twice must be bit-identical"
    for other in outs[2:]:
        for a, b in zip(outs[0], other):
            assert max_rel_err(b, a) < 2e-2


# ---------------------------------------------------------------- boundary behaviour


def test_state_init_zeroes():
    layer = GpuLayer(2, 3, 64, "bf16", "bf16")
    S1, S2 = layer.states()
    assert not S1.any() and not S2.any()


def test_T0_is_noop_and_errors_do_nothing():
    import torch
    import paper_2506_09316_amd as dsla
    layer = GpuLayer(1, 2, 64, "f32", "f32")
    S10, S20 = wl.initial_states(3, 1, 2, 64, 64)
    layer.set_states(S10, S20)
    dsla.dsla_prefill(layer.desc, 0, None, None, None, None, None, layer.S1, layer.S2, None, None)
    with pytest.raises(dsla.DslaError) as e:
        q = torch.zeros(1, 8, 2, 64, device="cuda")
        dsla.dsla_prefill(layer.desc, 8, q, q, q, q, None, layer.S1, layer.S2, q, None)
    assert e.value.status == 1
    torch.cuda.synchronize()
    S1, S2 = layer.states()
    assert np.array_equal(S1, S10) and np.array_equal(S2, S20)


def test_random_configurations():
    """Forty seeded random small configurations of the dense entry points: head size, storage types, chunk, segment
    count, sequence length (ragged against both), batch, heads, blend factor (also outside [0, 1]), scale, gate mode,
    carried-in states, a continuation call and decode steps, each against the oracle."""
    rng = np.random.default_rng(20250609)
    for case in range(40):
        d = int(rng.choice([64, 128]))
        io = str(rng.choice(["bf16", "f32"]))
        gate = str(rng.choice(["bf16", "f32"]))
        chunk = int(rng.choice([0, 32, 64, 128]))
        T = int(rng.integers(1, 330))
        segments = int(rng.integers(0, 6))
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        gamma = float(rng.choice([0.0, 0.25, 0.5, 0.8, 1.0, 1.4, -0.3]))
        scale = float(rng.choice([1.0, 0.5, -0.7]))
        mode = int(rng.integers(0, 2))
        steps = int(rng.integers(0, 3))
        tol = 1e-4 if io == "f32" else 2e-2
        print(f"  case {case}: d={d} io={io} gate={gate} chunk={chunk} T={T} segments={segments} B={B} H={H} "
              f"gamma={gamma} scale={scale} gate_mode={mode} decode={steps}", flush=True)
        x = wl.layer_inputs(1000 + case, B, T + steps, H, d, d, io_dtype=io, gate_dtype=gate, qk_scale=d ** -0.5,
                            gates="preact" if mode else "log")
        g1, g2 = ((orc.log_gates_from_preactivations(x[n], 16.0) for n in ("g1", "g2")) if mode else (x["g1"], x["g2"]))
        S1_0, S2_0 = wl.initial_states(2000 + case, B, H, d, d, amplitude=0.3)
        layer = GpuLayer(B, H, d, io, gate, gamma=gamma, scale=scale, chunk=chunk, segments=segments, gate_mode=mode)
        layer.set_states(S1_0, S2_0)
        cut = int(rng.integers(0, T + 1))
        outs = []
        if cut:
            outs.append(layer.prefill(slice_t(x, 0, cut)))
        if cut < T:
            outs.append(layer.prefill(slice_t(x, cut, T)))
        for t in range(T, T + steps):
            outs.append(layer.decode(slice_t(x, t, t + 1)))
        o = np.concatenate(outs, 1)
        S1, S2 = layer.states()
        ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], g1, g2, gamma, scale, S1=S1_0, S2=S2_0)
        assert np.all(np.isfinite(o))
        for name, got, ref in (("o", o, ro), ("S1", S1, rS1), ("S2", S2, rS2)):
            err = max_rel_err(got, ref)
            assert err <= tol, f"case {case} {name}: {err:.3e} > {tol}"

