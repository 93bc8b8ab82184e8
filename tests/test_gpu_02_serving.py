"""GPU parity of the serving-side entry points: gate pre-activations applied in the kernels, packed sequences of
different lengths, the state pool and sub-batches served in place, each against the CPU oracle."""
import numpy as np
import pytest

from oracle import dsla_oracle as orc
import workloads as wl
import paper_2506_09316_amd as dsla
from tests.gpu_common import TOL, check
from tests.util import GpuLayer, code, max_rel_err, slice_t, to_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("io,gate,d,T,tau,tol", [("bf16", "bf16", 128, 1500, 16.0, 2e-2), ("bf16", "f32", 64, 700, 16.0, 2e-2),
                                                 ("f32", "f32", 64, 520, 16.0, 1e-4), ("f32", "f32", 128, 300, 1.0, 1e-4),
                                                 ("f32", "bf16", 128, 200, 4.0, 1e-4)])
def test_gate_preactivation_mode(io, gate, d, T, tau, tol):
    """The gate tensors hold pre-activations z and the kernels form log alpha themselves; the oracle gets
    log alpha from its own map of the same (storage-rounded) z.  Prefill, a continuation call, and decode
    steps; the z of a few tokens are pushed far out (|z| up to 30) to cover both asymptotes of the map."""
    B, H, steps = 2, 3, 5
    x = wl.layer_inputs(77, B, T + steps, H, d, d, io_dtype=io, gate_dtype=gate, gates="preact", qk_scale=d ** -0.5,
                        gate_mean=2.0 if tau > 1 else 4.0)
    for n, sign in (("g1", 1.0), ("g2", -1.0)):
        x[n][:, 5::97] = np.float32(30.0 * sign) if tau > 1 else np.float32(30.0)
        x[n][:, 11::131, :, ::7] = np.float32(-6.0) if tau > 1 else np.float32(-2.0)
    lg = {n: orc.log_gates_from_preactivations(x[n], tau) for n in ("g1", "g2")}
    C = 64
    layer = GpuLayer(B, H, d, io, gate, gamma=0.35, chunk=C, gate_mode=1, tau=tau)
    T1 = 2 * T // 3 + 5
    outs = [layer.prefill(slice_t(x, 0, T1)), layer.prefill(slice_t(x, T1, T))]
    for t in range(T, T + steps):
        outs.append(layer.decode(slice_t(x, t, t + 1)))
    o = np.concatenate(outs, 1)
    S1, S2 = layer.states()
    ro, rS1, rS2 = orc.recurrent(x["q"], x["k"], x["v"], lg["g1"], lg["g2"], 0.35)
    check("o prefill", o[:, :T], ro[:, :T], tol)
    check("o decode", o[:, T:], ro[:, T:], tol)
    check("S1", S1, rS1, tol)
    check("S2", S2, rS2, tol)


def _run_varlen(lengths, H, d, io, gate, tol, *, slots=None, n_slots=None, segments=0, chunk=64, seed=91, decode_steps=0,
                max_T=None):
    """Packed prefill of sequences with the given lengths (and optionally decode steps on the same state pool),
    each sequence checked against the oracle run on it alone; pool entries no sequence names must stay bit-equal."""
    import torch
    B = len(lengths)
    total = int(sum(lengths))
    n_slots = n_slots or B
    slots = list(range(B)) if slots is None else list(slots)
    x = wl.layer_inputs(seed, 1, total + decode_steps * B, H, d, d, io_dtype=io, gate_dtype=gate, qk_scale=d ** -0.5)
    S1_0, S2_0 = wl.initial_states(seed, n_slots, H, d, d, amplitude=0.3)
    desc = dsla.make_desc(B, H, d, d, io_dtype=code(io), gate_dtype=code(gate), gamma=0.6, chunk=chunk, segments=segments)
    S1, S2 = (torch.from_numpy(a.copy()).cuda() for a in (S1_0, S2_0))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    cu_t = torch.from_numpy(cu).cuda()
    slot_t = torch.tensor(slots, dtype=torch.int32, device="cuda")
    q, k, v = (to_gpu(x[n][0, :total], io) for n in ("q", "k", "v"))
    g1, g2 = (to_gpu(x[n][0, :total], gate) for n in ("g1", "g2"))
    o = torch.full_like(v, float("nan"))
    mT = max(lengths) if max_T is None else max_T
    nbytes = dsla.dsla_prefill_varlen_workspace_bytes(desc, total, mT)
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda") if nbytes else None
    dsla.dsla_prefill_varlen(desc, total, mT, cu_t, slot_t, q, k, v, g1, g2, S1, S2, o, ws)
    outs_dec = []
    for s in range(decode_steps):
        a, b = total + s * B, total + (s + 1) * B
        dq, dk_, dv_ = (to_gpu(x[n][0, a:b], io) for n in ("q", "k", "v"))
        dg1, dg2 = (to_gpu(x[n][0, a:b], gate) for n in ("g1", "g2"))
        do = torch.full_like(dv_, float("nan"))
        dsla.dsla_decode_slots(desc, dq, dk_, dv_, dg1, dg2, slot_t, S1, S2, do)
        outs_dec.append(do.float().cpu().numpy())
    torch.cuda.synchronize()
    o = o.float().cpu().numpy()
    S1, S2 = S1.cpu().numpy(), S2.cpu().numpy()
    for b, L in enumerate(lengths):
        sl = slots[b]
        rows = list(range(cu[b], cu[b + 1])) + [total + s * B + b for s in range(decode_steps)]
        xs = {n: x[n][:, rows] for n in x}
        ro, rS1, rS2 = orc.recurrent(xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], 0.6,
                                     S1=S1_0[sl:sl + 1], S2=S2_0[sl:sl + 1])
        if L:
            check(f"o[seq {b}, {L} tokens]", o[cu[b]:cu[b + 1]][None], ro[:, :L], tol)
        for s in range(decode_steps):
            check(f"o decode[seq {b}, step {s}]", outs_dec[s][b][None, None], ro[:, L + s:L + s + 1], tol)
        check(f"S1[seq {b}]", S1[sl:sl + 1], rS1, tol)
        check(f"S2[seq {b}]", S2[sl:sl + 1], rS2, tol)
    for sl in set(range(n_slots)) - set(slots):
        assert np.array_equal(S1[sl], S1_0[sl]) and np.array_equal(S2[sl], S2_0[sl]), f"pool entry {sl} was touched"
    assert np.all(np.isfinite(o))


def test_varlen_fp32_ragged_lengths_one_segment():
    _run_varlen([1, 31, 32, 33, 0, 200, 64, 97], 2, 64, "f32", "f32", 1e-4)


def test_varlen_fp32_segments_differ_per_sequence():
    # longest sequence cut into 5 segments of 128 tokens; the others use 0, 1, 2, 5 and 3 of them, one ends on a boundary
    _run_varlen([600, 0, 100, 256, 513, 300], 2, 64, "f32", "f32", 1e-4, segments=5)
    _run_varlen([130, 640, 7], 1, 128, "f32", "f32", 1e-4, segments=5, chunk=32, max_T=640)


def test_varlen_bf16_state_pool_and_decode():
    # serving shape in miniature: 5 requests in a pool of 9 state entries, prompts of mixed length, then 3 decode steps
    _run_varlen([700, 45, 1300, 1, 256], 3, 128, "bf16", "bf16", 2e-2, slots=[7, 2, 0, 8, 4], n_slots=9, decode_steps=3)
    _run_varlen([513, 2100], 2, 64, "bf16", "f32", 2e-2, slots=[1, 0], n_slots=3, segments=0, decode_steps=1, max_T=2500)


def test_varlen_many_sequences():
    """More sequences than the list-building workgroup has threads (each thread then takes a run of sequences),
    most of them a few tokens long, a few long enough to be cut into segments."""
    rng = np.random.default_rng(5)
    lengths = [int(x) for x in rng.integers(0, 40, size=300)]
    for at, L in ((3, 900), (150, 1300), (299, 517)):
        lengths[at] = L
    _run_varlen(lengths, 1, 64, "bf16", "bf16", 2e-2, segments=6, chunk=32, seed=93)


def test_varlen_gate_preactivations():
    import torch
    lengths, H, d, tau = [300, 77, 1, 640], 2, 128, 16.0
    B, total = len(lengths), sum(lengths)
    x = wl.layer_inputs(95, 1, total, H, d, d, io_dtype="bf16", gate_dtype="bf16", gates="preact", qk_scale=d ** -0.5)
    lg = {n: orc.log_gates_from_preactivations(x[n], tau) for n in ("g1", "g2")}
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.3, chunk=64, segments=3,
                          gate_mode=1, tau=tau)
    S1 = torch.zeros(B, H, d, d, device="cuda"); S2 = torch.zeros_like(S1)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    t = {n: to_gpu(x[n][0], "bf16") for n in x}
    o = torch.full_like(t["v"], float("nan"))
    ws = torch.empty(max(dsla.dsla_prefill_varlen_workspace_bytes(desc, total, max(lengths)), 1), dtype=torch.uint8, device="cuda")
    dsla.dsla_prefill_varlen(desc, total, max(lengths), torch.from_numpy(cu).cuda(), None, t["q"], t["k"], t["v"], t["g1"],
                             t["g2"], S1, S2, o, ws)
    torch.cuda.synchronize()
    o = o.float().cpu().numpy()
    for b in range(B):
        sl = slice(cu[b], cu[b + 1])
        ro, rS1, rS2 = orc.recurrent(x["q"][:, sl], x["k"][:, sl], x["v"][:, sl], lg["g1"][:, sl], lg["g2"][:, sl], 0.3)
        check(f"o[seq {b}]", o[sl][None], ro, 2e-2)
        check(f"S1[seq {b}]", S1[b:b + 1].cpu().numpy(), rS1, 2e-2)
        check(f"S2[seq {b}]", S2[b:b + 1].cpu().numpy(), rS2, 2e-2)


def test_sub_batch_served_in_place():
    """A mixed batch of 7 requests of which 4 use the DSLA form of this layer: the prefill names them through
    seq_index, the decode step through row_index, their states live in a pool.  Each is checked against the oracle
    run on it alone; the output rows of the other requests must keep the bytes they had."""
    import torch
    lengths, H, d = [120, 700, 33, 0, 1500, 64, 257], 2, 128
    dsla_seqs = [4, 1, 6, 2]          # participating requests, in the order this call lists them
    slots, n_slots = [5, 0, 3, 2], 6
    B_all, total = len(lengths), sum(lengths)
    x = wl.layer_inputs(97, 1, total + B_all, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=d ** -0.5)
    S1_0, S2_0 = wl.initial_states(97, n_slots, H, d, d, amplitude=0.3)
    S1, S2 = (torch.from_numpy(a.copy()).cuda() for a in (S1_0, S2_0))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    desc = dsla.make_desc(len(dsla_seqs), H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.45, chunk=64,
                          segments=4)
    t = {n: to_gpu(x[n][0, :total], "bf16") for n in x}
    marker = 1.5
    o = torch.full_like(t["v"], marker)
    max_T = max(lengths[i] for i in dsla_seqs)
    ws = torch.empty(dsla.dsla_prefill_varlen_workspace_bytes(desc, total, max_T), dtype=torch.uint8, device="cuda")
    seq_t = torch.tensor(dsla_seqs, dtype=torch.int32, device="cuda")
    slot_t = torch.tensor(slots, dtype=torch.int32, device="cuda")
    dsla.dsla_prefill_varlen(desc, total, max_T, torch.from_numpy(cu).cuda(), slot_t, t["q"], t["k"], t["v"], t["g1"],
                             t["g2"], S1, S2, o, ws, seq_index=seq_t)
    # one decode token for every request of the batch lies in rows total .. total + B_all - 1; only the DSLA ones are served
    dt = {n: to_gpu(x[n][0, total:], "bf16") for n in x}
    do = torch.full_like(dt["v"], marker)
    dsla.dsla_decode_slots(desc, dt["q"], dt["k"], dt["v"], dt["g1"], dt["g2"], slot_t, S1, S2, do, row_index=seq_t)
    torch.cuda.synchronize()
    o, do = o.float().cpu().numpy(), do.float().cpu().numpy()
    S1, S2 = S1.cpu().numpy(), S2.cpu().numpy()
    for b, (sq, sl) in enumerate(zip(dsla_seqs, slots)):
        rows = list(range(cu[sq], cu[sq + 1])) + [total + sq]
        xs = {n: x[n][:, rows] for n in x}
        ro, rS1, rS2 = orc.recurrent(xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], 0.45, S1=S1_0[sl:sl + 1], S2=S2_0[sl:sl + 1])
        L = lengths[sq]
        check(f"o[request {sq}]", o[cu[sq]:cu[sq + 1]][None], ro[:, :L], 2e-2)
        check(f"o decode[request {sq}]", do[sq][None, None], ro[:, L:], 2e-2)
        check(f"S1[request {sq}]", S1[sl:sl + 1], rS1, 2e-2)
        check(f"S2[request {sq}]", S2[sl:sl + 1], rS2, 2e-2)
    for sq in set(range(B_all)) - set(dsla_seqs):
        assert np.all(o[cu[sq]:cu[sq + 1]] == marker) and np.all(do[sq] == marker), f"rows of request {sq} were written"
    for sl in set(range(n_slots)) - set(slots):
        assert np.array_equal(S1[sl], S1_0[sl]) and np.array_equal(S2[sl], S2_0[sl])


def test_varlen_equals_dense_bitwise():
    """Equal lengths, identity slots: the packed entry point runs the same kernels with the same segment length
    (its workgroups find their segments through the device-built lists instead of their index)."""
    import torch
    B, T, H, d = 3, 384, 2, 128
    x = wl.layer_inputs(17, B, T, H, d, d, io_dtype="bf16", gate_dtype="bf16", qk_scale=d ** -0.5)
    layer = GpuLayer(B, H, d, "bf16", "bf16", gamma=0.6, chunk=64, segments=3)
    o_dense = layer.prefill(x)
    S1d, S2d = layer.states()
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.6, chunk=64, segments=3)
    S1 = torch.zeros(B, H, d, d, device="cuda"); S2 = torch.zeros_like(S1)
    cu = torch.arange(0, (B + 1) * T, T, dtype=torch.int32, device="cuda")
    t = {n: to_gpu(x[n].reshape(B * T, H, d), "bf16") for n in x}
    o = torch.full_like(t["v"], float("nan"))
    nbytes = dsla.dsla_prefill_varlen_workspace_bytes(desc, B * T, T)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dsla.dsla_prefill_varlen(desc, B * T, T, cu, None, t["q"], t["k"], t["v"], t["g1"], t["g2"], S1, S2, o, ws)
    torch.cuda.synchronize()
    assert np.array_equal(o.float().cpu().numpy().reshape(B, T, H, d), o_dense)
    assert np.array_equal(S1.cpu().numpy(), S1d) and np.array_equal(S2.cpu().numpy(), S2d)



# ---------------------------------------------------------------- projections in front of the layer
def _projection_case(seed, M, K, n_out, width, bias):
    rng = np.random.default_rng(seed)
    x = wl.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    W = wl.round_to_bf16(rng.standard_normal((n_out * width, K), dtype=np.float32) * np.float32(K ** -0.5))
    b = rng.standard_normal(n_out * width).astype(np.float32) if bias else None
    return x, W, b


@pytest.mark.parametrize("M,K,n_out,width,bias", [(300, 256, 5, 256, False), (128, 64, 1, 128, True), (1000, 512, 3, 384, True),
                                                  (1, 32, 2, 128, False), (4096, 1024, 5, 1024, False),
                                                  (513, 128, 1, 128, True), (256, 384, 2, 256, True), (700, 96, 2, 128, False)])
def test_project_against_library_matmul(M, K, n_out, width, bias):
    """dsla_project against the definition through a library matmul in fp64 on the same bf16 inputs; the results are
    stored as bf16, so an element may differ from the exact product by half a bf16 unit of itself plus the fp32
    accumulation error of K terms."""
    import torch
    x, W, b = _projection_case(800 + M, M, K, n_out, width, bias)
    outs = [torch.full((M, width), float("nan"), device="cuda", dtype=torch.bfloat16) for _ in range(n_out)]
    dsla.dsla_project(to_gpu(x, "bf16"), to_gpu(W, "bf16"), outs, torch.from_numpy(b).cuda() if bias else None)
    torch.cuda.synchronize()
    ref = x.astype(np.float64) @ W.astype(np.float64).T + (b.astype(np.float64) if bias else 0.0)
    for j in range(n_out):
        got = outs[j].float().cpu().numpy()
        r = ref[:, j * width:(j + 1) * width]
        assert np.all(np.isfinite(got))
        assert np.max(np.abs(got - r) / (np.abs(r) + 1e-2 * np.max(np.abs(r)))) <= 2 ** -8 * 1.1, f"output {j}"


def test_projections_feed_the_prefill():
    """The layer from its input: x -> one GEMM -> q, k, v and the two gate pre-activations in the prefill's own
    layout -> dsla_prefill with gate_mode = DSLA_GATE_PREACT.  The oracle takes the same bf16 weights and input
    through a library matmul (fp64), rounds the five tensors to bf16 as the GPU stores them, maps the gates and runs
    the recurrence.  The history gate's weight is a scaled identity plus noise, the recency gate's is random, as the
    paper initialises them."""
    import torch
    B, T, H, d, tau = 2, 300, 2, 128, 16.0
    Dm = H * d
    rng = np.random.default_rng(820)
    x = wl.round_to_bf16(rng.standard_normal((B * T, Dm), dtype=np.float32))
    Wq, Wk, Wv = (rng.standard_normal((Dm, Dm), dtype=np.float32) * np.float32(Dm ** -0.5 * d ** -0.25) for _ in range(3))
    Wg1 = np.eye(Dm, dtype=np.float32) * 2.0 + rng.standard_normal((Dm, Dm), dtype=np.float32) * np.float32(0.02)
    Wg2 = rng.standard_normal((Dm, Dm), dtype=np.float32) * np.float32(Dm ** -0.5)
    W = wl.round_to_bf16(np.concatenate([Wq, Wk, Wv, Wg1, Wg2]))
    outs = [torch.empty(B, T, H, d, device="cuda", dtype=torch.bfloat16) for _ in range(5)]
    dsla.dsla_project(to_gpu(x, "bf16"), to_gpu(W, "bf16"), outs)
    desc = dsla.make_desc(B, H, d, d, io_dtype=code("bf16"), gate_dtype=code("bf16"), gamma=0.4, chunk=64, gate_mode=1, tau=tau,
                          zero_init=True)
    S1 = torch.full((B, H, d, d), float("nan"), device="cuda")
    S2 = torch.full_like(S1, float("nan"))
    o = torch.full_like(outs[2], float("nan"))
    nbytes = dsla.dsla_prefill_workspace_bytes(desc, T)
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")
    dsla.dsla_prefill(desc, T, outs[0], outs[1], outs[2], outs[3], outs[4], S1, S2, o, ws if nbytes else None)
    torch.cuda.synchronize()
    y = wl.round_to_bf16((x.astype(np.float64) @ W.astype(np.float64).T).astype(np.float32)).reshape(B, T, 5, H, d)
    q, k, v, z1, z2 = (y[:, :, j] for j in range(5))
    ro, rS1, rS2 = orc.recurrent(q, k, v, orc.log_gates_from_preactivations(z1, tau), orc.log_gates_from_preactivations(z2, tau), 0.4)
    check("o", o.float().cpu().numpy(), ro, 2e-2)
    check("S1", S1.cpu().numpy(), rS1, 2e-2)
    check("S2", S2.cpu().numpy(), rS2, 2e-2)
