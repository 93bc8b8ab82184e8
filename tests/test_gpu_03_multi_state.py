"""GPU parity of the calls for N states, the outer-product gate and grouped key/value heads (dsla_decode_multi,
dsla_prefill_multi) against the CPU oracle's nstate recurrence."""
import numpy as np
import pytest

from oracle import dsla_oracle as orc
import workloads as wl
import paper_2506_09316_amd as dsla
from tests.gpu_common import TOL, check
from tests.util import code, to_gpu

pytestmark = pytest.mark.gpu


def _inputs(seed, N, B, T, H, Hkv, d, io, gd, beta):
    """q [B,T,H,d]; k, v [B,T,Hkv,d]; log-gates alpha [N,B,T,H,d] (state n forgets faster than state n-1) and beta."""
    x = wl.layer_inputs(seed, B, T, H, d, d, io_dtype=io, gate_dtype=gd, qk_scale=d ** -0.5)
    kv = wl.layer_inputs(seed + 7, B, T, Hkv, d, d, io_dtype=io, gate_dtype=gd, qk_scale=d ** -0.5)
    ga = np.stack([wl.layer_inputs(seed + 20 + n, B, T, H, d, d, io_dtype=io, gate_dtype=gd, tau=16.0 / (1 + n))["g1"]
                   for n in range(N)])
    gb = None
    if beta:
        gb = np.stack([wl.layer_inputs(seed + 40 + n, B, T, H, d, d, io_dtype=io, gate_dtype=gd, tau=24.0)["g2"]
                       for n in range(N)])
    w = np.random.default_rng(seed + 60).uniform(-0.3, 1.0, N).astype(np.float32)
    S0 = np.stack([wl.initial_states(seed + 70 + n, B, H, d, d, amplitude=0.3)[0] for n in range(N)])
    return x["q"], kv["k"], kv["v"], ga, gb, w, S0


@pytest.mark.parametrize("N,Hkv,beta,io,gd,d", [(1, 4, False, "f32", "f32", 64), (2, 4, True, "bf16", "bf16", 128),
                                                 (4, 2, True, "f32", "f32", 128), (8, 1, True, "bf16", "f32", 64),
                                                 (3, 4, False, "bf16", "bf16", 128)])
def test_decode_multi(N, Hkv, beta, io, gd, d):
    import torch
    B, H, steps = 3, 4, 5
    q, k, v, ga, gb, w, S0 = _inputs(300 + N, N, B, steps, H, Hkv, d, io, gd, beta)
    desc = dsla.make_desc(B, H, d, d, io_dtype=code(io), gate_dtype=code(gd), scale=0.8)
    S = [torch.from_numpy(S0[n].copy()).cuda() for n in range(N)]
    Sref = S0.astype(np.float64)
    for t in range(steps):
        tq, tk, tv = to_gpu(q[:, t], io), to_gpu(k[:, t], io), to_gpu(v[:, t], io)
        tga = [to_gpu(ga[n][:, t], gd) for n in range(N)]
        tgb = [to_gpu(gb[n][:, t], gd) for n in range(N)] if beta else None
        o = torch.full((B, H, d), float("nan"), device="cuda", dtype=tq.dtype)
        multi = dsla.make_multi(tga, S, w, g_beta=tgb, H_kv=Hkv)
        dsla.dsla_decode_multi(desc, multi, tq, tk, tv, o)
        torch.cuda.synchronize()
        ro, Sref = orc.nstate(q[:, t:t + 1], k[:, t:t + 1], v[:, t:t + 1], ga[:, :, t:t + 1],
                              gb[:, :, t:t + 1] if beta else None, w, 0.8, S=Sref)
        check(f"o[{t}]", o.float().cpu().numpy()[:, None], ro, TOL[io])
    for n in range(N):
        check(f"S[{n}]", S[n].cpu().numpy(), Sref[n], 1e-5)


def test_decode_multi_equals_decode_for_two_states():
    """N = 2, no beta gate, H_kv = H, blend (gamma, 1 - gamma): the same numbers as dsla_decode."""
    import torch
    B, H, d, gamma = 2, 3, 128, 0.35
    q, k, v, ga, _, _, S0 = _inputs(320, 2, B, 1, H, H, d, "bf16", "bf16", False)
    t = [to_gpu(a[:, 0], "bf16") for a in (q, k, v, ga[0], ga[1])]
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=gamma)
    Sa = [torch.from_numpy(S0[n].copy()).cuda() for n in range(2)]
    Sb = [torch.from_numpy(S0[n].copy()).cuda() for n in range(2)]
    oa, ob = torch.empty_like(t[2]), torch.empty_like(t[2])
    dsla.dsla_decode(desc, t[0], t[1], t[2], t[3], t[4], Sa[0], Sa[1], oa)
    dsla.dsla_decode_multi(desc, dsla.make_multi([t[3], t[4]], Sb, [gamma, 1.0 - gamma]), t[0], t[1], t[2], ob)
    torch.cuda.synchronize()
    assert torch.equal(Sa[0], Sb[0]) and torch.equal(Sa[1], Sb[1])
    np.testing.assert_allclose(ob.float().cpu().numpy(), oa.float().cpu().numpy(), rtol=2 ** -7, atol=1e-6)


@pytest.mark.parametrize("N,Hkv,io,gd,d,T,segments,beta", [
    (1, 2, "f32", "f32", 64, 200, 2, ()), (2, 1, "bf16", "bf16", 128, 700, 3, ()), (3, 4, "f32", "f32", 64, 333, 1, ()),
    (4, 2, "bf16", "bf16", 128, 1100, 0, ()), (4, 4, "f32", "bf16", 128, 150, 2, ()), (8, 2, "bf16", "f32", 64, 450, 2, ()),
    (1, 4, "f32", "f32", 64, 300, 2, (0,)), (1, 4, "bf16", "bf16", 128, 500, 3, (0,)), (2, 2, "f32", "f32", 128, 170, 1, (0, 1)),
    (3, 1, "bf16", "bf16", 128, 900, 2, (1,)), (4, 4, "bf16", "f32", 64, 257, 2, (0, 3)), (2, 4, "f32", "f32", 64, 31, 1, (1,)),
    # plans of the library's own with two segments: the pre-pass works on the halves of the first one
    (3, 2, "bf16", "bf16", 128, 700, 0, (1,)), (2, 4, "f32", "f32", 64, 700, 0, (0,))])
def test_prefill_multi(N, Hkv, io, gd, d, T, segments, beta):
    """N states through the prefill kernels (two at a time without a beta gate, one at a time with one), grouped
    key/value heads, carried-in states, then a decode step on the same states.  `beta` lists the states that have a
    beta gate (the outer-product gate alpha^T beta of the background section)."""
    import torch
    B, H = 2, 4
    q, k, v, ga, gb, w, S0 = _inputs(340 + N, N, B, T + 1, H, Hkv, d, io, gd, bool(beta))
    if beta:
        for n in range(N):
            if n not in beta:
                gb[n] = 0.0          # the oracle's beta = 1 for the states that have no such gate
    desc = dsla.make_desc(B, H, d, d, io_dtype=code(io), gate_dtype=code(gd), scale=0.9, chunk=64, segments=segments)
    S = [torch.from_numpy(S0[n].copy()).cuda() for n in range(N)]
    tq, tk, tv = to_gpu(q[:, :T], io), to_gpu(k[:, :T], io), to_gpu(v[:, :T], io)
    tga = [to_gpu(ga[n][:, :T], gd) for n in range(N)]
    tgb = [to_gpu(gb[n][:, :T], gd) if n in beta else None for n in range(N)] if beta else None
    multi = dsla.make_multi(tga, S, w, g_beta=tgb, H_kv=Hkv)
    o = torch.full((B, T, H, d), float("nan"), device="cuda", dtype=tq.dtype)
    nbytes = dsla.dsla_prefill_multi_workspace_bytes(desc, multi, T)
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")
    dsla.dsla_prefill_multi(desc, multi, T, tq, tk, tv, o, ws)
    dq, dk_, dv_ = to_gpu(q[:, T], io), to_gpu(k[:, T], io), to_gpu(v[:, T], io)
    dga = [to_gpu(ga[n][:, T], gd) for n in range(N)]
    dgb = [to_gpu(gb[n][:, T], gd) if n in beta else None for n in range(N)] if beta else None
    do = torch.full((B, H, d), float("nan"), device="cuda", dtype=tq.dtype)
    dsla.dsla_decode_multi(desc, dsla.make_multi(dga, S, w, g_beta=dgb, H_kv=Hkv), dq, dk_, dv_, do)
    torch.cuda.synchronize()
    ro, rS = orc.nstate(q, k, v, ga, gb if beta else None, w, 0.9, S=S0)
    tol = TOL[io]
    check("o prefill", o.float().cpu().numpy(), ro[:, :T], tol)
    check("o decode", do.float().cpu().numpy()[:, None], ro[:, T:], tol)
    for n in range(N):
        check(f"S[{n}]", S[n].cpu().numpy(), rS[n], tol)


def test_prefill_multi_beta_gate_with_strong_column_decay():
    """A beta gate as strong as plain-sigmoid gates with pre-activations around -1 (tau = 1): the decay of a column over a
    32-token step spans tens of binary orders of magnitude, which the centred split between the values and the output
    has to carry; status stays clear."""
    import torch
    B, T, H, d = 1, 200, 2, 64
    q, k, v, ga, gb, w, S0 = _inputs(380, 1, B, T, H, H, d, "f32", "f32", True)
    gb[0] = wl.layer_inputs(381, B, T, H, d, d, io_dtype="f32", gate_dtype="f32", tau=1.0, gate_mean=-1.0)["g2"]
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("f32"), gate_dtype=code("f32"), chunk=64, segments=2, status=status)
    S = [torch.from_numpy(S0[0].copy()).cuda()]
    multi = dsla.make_multi([to_gpu(ga[0], "f32")], S, w, g_beta=[to_gpu(gb[0], "f32")])
    o = torch.full((B, T, H, d), float("nan"), device="cuda")
    ws = torch.empty(max(dsla.dsla_prefill_multi_workspace_bytes(desc, multi, T), 1), dtype=torch.uint8, device="cuda")
    dsla.dsla_prefill_multi(desc, multi, T, to_gpu(q, "f32"), to_gpu(k, "f32"), to_gpu(v, "f32"), o, ws)
    torch.cuda.synchronize()
    ro, rS = orc.nstate(q, k, v, ga, gb, w, 1.0, S=S0)
    check("o", o.cpu().numpy(), ro, 1e-4)
    check("S", S[0].cpu().numpy(), rS[0], 1e-4)
    assert int(status.item()) == 0


def test_multi_state_argument_checks():
    import torch
    B, H, d, T = 1, 2, 64, 64
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("f32"), gate_dtype=code("f32"))
    z = torch.zeros(B, T, H, d, device="cuda")
    S = [torch.zeros(B, H, d, d, device="cuda") for _ in range(2)]
    with pytest.raises(dsla.DslaError) as e:      # the prefill needs its workspace
        dsla.dsla_prefill_multi(desc, dsla.make_multi([z, z], S, [0.5, 0.5]), T, z, z, z, z.clone(), None)
    assert e.value.status == 4
    with pytest.raises(dsla.DslaError) as e:      # H_kv must divide H
        dsla.dsla_decode_multi(desc, dsla.make_multi([z[:, 0], z[:, 0]], S, [0.5, 0.5], H_kv=3), z[:, 0], z[:, 0], z[:, 0], z[:, 0].clone())
    assert e.value.status == 2
    with pytest.raises(dsla.DslaError) as e:      # two states in one buffer
        dsla.dsla_decode_multi(desc, dsla.make_multi([z[:, 0], z[:, 0]], [S[0], S[0]], [0.5, 0.5]), z[:, 0], z[:, 0], z[:, 0], z[:, 0].clone())
    assert e.value.status == 2
