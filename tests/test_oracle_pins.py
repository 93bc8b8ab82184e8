"""Pins of the CPU oracle against what the paper's equations and the mathematics fix.

None of these call the GPU library.  Each check is chosen so that a plausible mistake
in oracle/dsla_oracle.c (dropped term, wrong gate on a state, transposed operand,
read-out before the update, off-by-one in the gate product) fails at least one.
"""
import os

import numpy as np
import pytest

from oracle import dsla_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def rand_case(seed, B=2, T=13, H=3, dk=5, dv=4, strong=False):
    q, k = rnd(seed, B, T, H, dk), rnd(seed + 1, B, T, H, dk)
    v = rnd(seed + 2, B, T, H, dv)
    lo = 3.0 if strong else 0.3
    g1 = -np.random.default_rng(seed + 3).uniform(0.0, lo, (B, T, H, dk))
    g2 = -np.random.default_rng(seed + 4).uniform(0.0, 3 * lo, (B, T, H, dk))
    return q, k, v, g1, g2


def test_hand_example_d1():
    rows = np.loadtxt(os.path.join(GOLD, "hand_example_d1.txt"))
    T = rows.shape[0]
    one = np.ones((1, T, 1, 1))
    g1 = np.full((1, T, 1, 1), np.log(0.5))
    g2 = np.zeros((1, T, 1, 1))
    o, S1, S2 = orc.recurrent(one, one, one, g1, g2, 0.5)
    np.testing.assert_allclose(o.ravel(), rows[:, 3], rtol=0, atol=1e-15)
    assert S1.ravel()[0] == pytest.approx(rows[-1, 1], abs=1e-15)
    assert S2.ravel()[0] == pytest.approx(rows[-1, 2], abs=1e-15)
    # every prefix, through the state returned by a shorter call
    for t in range(T):
        _, s1, s2 = orc.recurrent(one[:, :t + 1], one[:, :t + 1], one[:, :t + 1], g1[:, :t + 1], g2[:, :t + 1], 0.5)
        assert s1.ravel()[0] == pytest.approx(rows[t, 1], abs=1e-15)
        assert s2.ravel()[0] == pytest.approx(rows[t, 2], abs=1e-15)
    np.testing.assert_allclose(orc.unrolled(one, one, one, g1, g2, 0.5).ravel(), rows[:, 3], atol=1e-15)


def test_hand_example_d2():
    rows = np.loadtxt(os.path.join(GOLD, "hand_example_d2.txt"))
    q = np.array([[1, 2], [2, -1]], float).reshape(1, 2, 1, 2)
    k = np.array([[1, 0], [2, 1]], float).reshape(1, 2, 1, 2)
    v = np.array([[3, 5], [1, -1]], float).reshape(1, 2, 1, 2)
    g1 = np.log(np.array([[0.5, 0.25], [0.5, 0.25]])).reshape(1, 2, 1, 2)
    g2 = np.log(np.array([[1.0, 0.5], [1.0, 0.5]])).reshape(1, 2, 1, 2)
    o, S1, S2 = orc.recurrent(q, k, v, g1, g2, 0.25)
    np.testing.assert_allclose(o.reshape(2, 2), rows[0:2], atol=1e-14)
    np.testing.assert_allclose(S1.reshape(2, 2), rows[2:4], atol=1e-14)
    np.testing.assert_allclose(S2.reshape(2, 2), rows[4:6], atol=1e-14)
    np.testing.assert_allclose(orc.unrolled(q, k, v, g1, g2, 0.25).reshape(2, 2), rows[0:2], atol=1e-14)


def test_ungated_is_causal_linear_attention():
    """log-gate 0 (alpha = 1): o = tril(Q K^T) V and S_T = K^T V, by library matmul."""
    B, T, H, dk, dv = 2, 17, 3, 6, 5
    q, k, v = rnd(1, B, T, H, dk), rnd(2, B, T, H, dk), rnd(3, B, T, H, dv)
    z = np.zeros((B, T, H, dk))
    o, S1, S2 = orc.recurrent(q, k, v, z, z, 0.3, scale=0.7)
    ou = orc.unrolled(q, k, v, z, z, 0.3, scale=0.7)
    for b in range(B):
        for h in range(H):
            Q, K, V = q[b, :, h], k[b, :, h], v[b, :, h]
            ref = 0.7 * np.tril(Q @ K.T) @ V
            np.testing.assert_allclose(o[b, :, h], ref, rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(ou[b, :, h], ref, rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(S1[b, h], K.T @ V, rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(S2[b, h], K.T @ V, rtol=1e-12, atol=1e-12)


def test_scalar_gate_is_decay_masked_matmul():
    """A gate that is the same for every feature: o = ((Q K^T) * D) V with
    D[t,s] = prod_{tau=s+1..t} a_tau for s <= t; the two states blend linearly."""
    B, T, H, dk, dv = 1, 19, 2, 4, 3
    q, k, v = rnd(4, B, T, H, dk), rnd(5, B, T, H, dk), rnd(6, B, T, H, dv)
    a1 = np.random.default_rng(7).uniform(0.5, 1.0, (B, T, H))
    a2 = np.random.default_rng(8).uniform(0.05, 0.9, (B, T, H))
    g1 = np.repeat(np.log(a1)[..., None], dk, -1)
    g2 = np.repeat(np.log(a2)[..., None], dk, -1)
    gam = 0.35
    o, _, _ = orc.recurrent(q, k, v, g1, g2, gam)
    for h in range(H):
        Q, K, V = q[0, :, h], k[0, :, h], v[0, :, h]

        def D(a):
            M = np.zeros((T, T))
            for t in range(T):
                for s in range(t + 1):
                    M[t, s] = np.prod(a[s + 1:t + 1])
            return M
        ref = ((Q @ K.T) * (gam * D(a1[0, :, h]) + (1 - gam) * D(a2[0, :, h]))) @ V
        np.testing.assert_allclose(o[0, :, h], ref, rtol=1e-11, atol=1e-12)


def test_geometric_closed_form():
    """Constant per-feature gate, constant k and v: S_T[d,:] = (1-a_d^T)/(1-a_d) k_d v."""
    T, dk, dv = 40, 4, 3
    a1 = np.array([0.9, 0.5, 1.0, 0.99])
    a2 = np.array([0.1, 0.7, 0.3, 1.0])
    kk, vv, qq = np.array([1.0, -2.0, 0.5, 3.0]), np.array([2.0, -1.0, 0.25]), np.array([0.3, 0.1, -0.7, 1.1])

    def tile(x):
        return np.broadcast_to(x, (1, T, 1, x.size)).copy()
    with np.errstate(divide="ignore"):
        o, S1, S2 = orc.recurrent(tile(qq), tile(kk), tile(vv), tile(np.log(a1)), tile(np.log(a2)), 0.6)

    def geo(a, n):
        return np.where(a == 1.0, float(n), (1 - a ** n) / np.where(a == 1.0, 1.0, 1 - a))
    np.testing.assert_allclose(S1[0, 0], (geo(a1, T) * kk)[:, None] * vv[None, :], rtol=1e-12)
    np.testing.assert_allclose(S2[0, 0], (geo(a2, T) * kk)[:, None] * vv[None, :], rtol=1e-12)
    for t in (0, 1, 7, T - 1):
        mix = 0.6 * geo(a1, t + 1) + 0.4 * geo(a2, t + 1)
        np.testing.assert_allclose(o[0, t, 0], np.sum(qq * kk * mix) * vv, rtol=1e-12)


def test_closed_gate_keeps_only_current_token():
    """alpha -> 0: S_t = k_t^T v_t and o_t = (q_t . k_t) v_t (read-out after the update,
    current token undecayed)."""
    B, T, H, dk, dv = 1, 6, 2, 3, 4
    q, k, v = rnd(9, B, T, H, dk), rnd(10, B, T, H, dk), rnd(11, B, T, H, dv)
    g = np.full((B, T, H, dk), -1.0e4)
    o, S1, S2 = orc.recurrent(q, k, v, g, g, 0.2)
    ref = np.einsum("bthd,bthd->bth", q, k)[..., None] * v
    np.testing.assert_allclose(o, ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S1[0, 1], np.outer(k[0, -1, 1], v[0, -1, 1]), rtol=1e-13)
    np.testing.assert_allclose(orc.unrolled(q, k, v, g, g, 0.2), ref, rtol=1e-13, atol=1e-13)


def test_recurrence_equals_unrolled_form():
    for seed, strong in ((100, False), (200, True)):
        q, k, v, g1, g2 = rand_case(seed, B=2, T=33, H=2, dk=7, dv=5, strong=strong)
        gam = np.array([0.3, 0.8])
        o, _, _ = orc.recurrent(q, k, v, g1, g2, gam, scale=1.3)
        ou = orc.unrolled(q, k, v, g1, g2, gam, scale=1.3)
        np.testing.assert_allclose(o, ou, rtol=1e-11, atol=1e-12)


def chunked_form(q, k, v, g1, g2, gamma, scale, C, S1, S2):
    """The recurrence of Section 4.1 regrouped C tokens at a time (test-side, numpy fp64, one (batch, head) pair):
    with b^i_r the sum of the log-gates of state i from the first token of the chunk up to token r,
        o_r  = scale * [ sum_i gamma_i (q_r * e^{b^i_r}) S^i  +  sum_{s <= r} w_{r,s} v_s ],
        w_rs = sum_d q_r[d] k_s[d] (gamma e^{b^1_r[d] - b^1_s[d]} + (1 - gamma) e^{b^2_r[d] - b^2_s[d]}),
        S^i <- diag(e^{b^i_C}) S^i + sum_s (k_s * e^{b^i_C - b^i_s})^T v_s,
    gamma_1 = gamma, gamma_2 = 1 - gamma.  q, k, g: [T, dk]; v: [T, dv]; S: [dk, dv]."""
    T = q.shape[0]
    S = [np.array(S1, dtype=np.float64), np.array(S2, dtype=np.float64)]
    gam = (gamma, 1.0 - gamma)
    o = np.zeros((T, v.shape[1]))
    for c0 in range(0, T, C):
        c1 = min(c0 + C, T)
        qc, kc, vc = q[c0:c1], k[c0:c1], v[c0:c1]
        w = np.zeros((c1 - c0, c1 - c0))
        carried = np.zeros((c1 - c0, v.shape[1]))
        for i, g in enumerate((g1, g2)):
            b = np.cumsum(g[c0:c1], axis=0)                                   # [r, d]
            carried += gam[i] * (qc * np.exp(b)) @ S[i]
            pair = np.exp(np.clip(b[:, None, :] - b[None, :, :], None, 0.0))  # [r, s, d]; only s <= r is used
            w += gam[i] * np.einsum("rd,sd,rsd->rs", qc, kc, pair)
            S[i] = np.exp(b[-1])[:, None] * S[i] + (kc * np.exp(b[-1][None, :] - b)).T @ vc
        o[c0:c1] = scale * (carried + np.tril(w) @ vc)
    return o, S[0], S[1]


@pytest.mark.parametrize("strong", [False, True])
def test_chunked_form_equals_recurrence(strong):
    """The chunked evaluation a prefill uses reaches the token-by-token recurrence for every chunk length,
    also when the length does not divide the sequence, with carried-in states."""
    B, T, H, dk, dv = 1, 150, 2, 6, 5
    q, k, v, g1, g2 = rand_case(900 + strong, B, T, H, dk, dv, strong=strong)
    S1 = rnd(911, B, H, dk, dv)
    S2 = rnd(912, B, H, dk, dv)
    for gamma, scale in ((0.3, 1.0), (1.4, -0.7)):
        ro, rS1, rS2 = orc.recurrent(q, k, v, g1, g2, gamma, scale, S1=S1, S2=S2)
        for C in (1, 2, 16, 64, 128, T, 7, 37):
            for h in range(H):
                o, s1, s2 = chunked_form(q[0, :, h], k[0, :, h], v[0, :, h], g1[0, :, h], g2[0, :, h], gamma, scale, C,
                                         S1[0, h], S2[0, h])
                np.testing.assert_allclose(o, ro[0, :, h], rtol=1e-11, atol=1e-11, err_msg=f"C={C}")
                np.testing.assert_allclose(s1, rS1[0, h], rtol=1e-11, atol=1e-11, err_msg=f"C={C}")
                np.testing.assert_allclose(s2, rS2[0, h], rtol=1e-11, atol=1e-11, err_msg=f"C={C}")


def test_brute_force_python_loops_tiny():
    """Quadruple loop over (t, s, d, j) with explicit gate products, tiny sizes."""
    q, k, v, g1, g2 = rand_case(300, B=1, T=6, H=1, dk=3, dv=2, strong=True)
    gam = 0.45
    o, _, _ = orc.recurrent(q, k, v, g1, g2, gam)
    a1, a2 = np.exp(g1), np.exp(g2)
    ref = np.zeros_like(o)
    for t in range(6):
        for s in range(t + 1):
            for d in range(3):
                p1 = p2 = 1.0
                for tau in range(s + 1, t + 1):
                    p1 *= a1[0, tau, 0, d]
                    p2 *= a2[0, tau, 0, d]
                for j in range(2):
                    ref[0, t, 0, j] += q[0, t, 0, d] * k[0, s, 0, d] * (gam * p1 + (1 - gam) * p2) * v[0, s, 0, j]
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-13)


def test_state_disabling_and_equal_gates():
    q, k, v, g1, g2 = rand_case(400)
    junk = -np.abs(rnd(401, *g1.shape))
    # gamma = 1: only the history state and its gate matter
    o1, S1a, _ = orc.recurrent(q, k, v, g1, g2, 1.0)
    o1b, S1b, _ = orc.recurrent(q, k, v, g1, junk, 1.0)
    np.testing.assert_allclose(o1, o1b, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S1a, S1b, rtol=0, atol=0)
    # gamma = 0: only the recency state and its gate matter
    o0, _, _ = orc.recurrent(q, k, v, g1, g2, 0.0)
    o0b, _, _ = orc.recurrent(q, k, v, junk, g2, 0.0)
    np.testing.assert_allclose(o0, o0b, rtol=1e-13, atol=1e-13)
    assert np.max(np.abs(o1 - o0)) > 1e-3  # the two single-state outputs do differ
    # single-state output with gate g equals gamma=1 with g1=g and gamma=0 with g2=g
    oa, _, _ = orc.recurrent(q, k, v, g1, junk, 1.0)
    ob, _, _ = orc.recurrent(q, k, v, junk, g1, 0.0)
    np.testing.assert_allclose(oa, ob, rtol=1e-13, atol=1e-13)
    # equal gates: output does not depend on gamma
    oc, _, _ = orc.recurrent(q, k, v, g1, g1, 0.15)
    od, _, _ = orc.recurrent(q, k, v, g1, g1, 0.9)
    np.testing.assert_allclose(oc, od, rtol=1e-12, atol=1e-12)
    # general gamma is the blend of the two single-state outputs
    og, _, _ = orc.recurrent(q, k, v, g1, g2, 0.37)
    np.testing.assert_allclose(og, 0.37 * o1 + 0.63 * o0, rtol=1e-12, atol=1e-12)


def test_linearity():
    q, k, v, g1, g2 = rand_case(500)
    v2, q2 = rnd(501, *v.shape), rnd(502, *q.shape)
    o, S1, S2 = orc.recurrent(q, k, v, g1, g2, 0.4)
    ov, S1v, _ = orc.recurrent(q, k, 2.0 * v - 3.0 * v2, g1, g2, 0.4)
    o2, S12, _ = orc.recurrent(q, k, v2, g1, g2, 0.4)
    np.testing.assert_allclose(ov, 2 * o - 3 * o2, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(S1v, 2 * S1 - 3 * S12, rtol=1e-11, atol=1e-11)
    oq, _, _ = orc.recurrent(q + q2, k, v, g1, g2, 0.4)
    oq2, _, _ = orc.recurrent(q2, k, v, g1, g2, 0.4)
    np.testing.assert_allclose(oq, o + oq2, rtol=1e-11, atol=1e-11)
    ok, S1k, _ = orc.recurrent(q, -1.5 * k, v, g1, g2, 0.4)
    np.testing.assert_allclose(ok, -1.5 * o, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(S1k, -1.5 * S1, rtol=1e-11, atol=1e-11)
    osc, _, _ = orc.recurrent(q, k, v, g1, g2, 0.4, scale=0.125)
    np.testing.assert_allclose(osc, 0.125 * o, rtol=1e-13, atol=1e-13)


def test_continuation_and_decode_steps():
    q, k, v, g1, g2 = rand_case(600, T=21)
    o, S1, S2 = orc.recurrent(q, k, v, g1, g2, 0.55)
    T1 = 8
    oa, s1, s2 = orc.recurrent(q[:, :T1], k[:, :T1], v[:, :T1], g1[:, :T1], g2[:, :T1], 0.55)
    outs = [oa]
    for t in range(T1, 21):  # decode: one token at a time on the carried states
        ot, s1, s2 = orc.recurrent(q[:, t:t + 1], k[:, t:t + 1], v[:, t:t + 1], g1[:, t:t + 1], g2[:, t:t + 1],
                                   0.55, S1=s1, S2=s2)
        outs.append(ot)
    np.testing.assert_allclose(np.concatenate(outs, 1), o, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(s1, S1, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(s2, S2, rtol=1e-13, atol=1e-13)


def test_initial_state_pure_decay():
    """k = 0: the carried-in state only decays, S_T = diag(prod alpha) S_0, o_t = q_t S_t."""
    B, T, H, dk, dv = 1, 9, 2, 4, 3
    q, _, _, g1, g2 = rand_case(700, B=B, T=T, H=H, dk=dk, dv=dv)
    S10, S20 = rnd(701, B, H, dk, dv), rnd(702, B, H, dk, dv)
    zk, zv = np.zeros((B, T, H, dk)), np.zeros((B, T, H, dv))
    o, S1, S2 = orc.recurrent(q, zk, zv, g1, g2, 0.25, S1=S10, S2=S20)
    c1, c2 = np.exp(np.cumsum(g1, 1)), np.exp(np.cumsum(g2, 1))  # [B,T,H,dk]
    np.testing.assert_allclose(S1[0], c1[0, -1][:, :, None] * S10[0], rtol=1e-12)
    np.testing.assert_allclose(S2[0], c2[0, -1][:, :, None] * S20[0], rtol=1e-12)
    for t in (0, 4, T - 1):
        for h in range(H):
            mix = 0.25 * c1[0, t, h][:, None] * S10[0, h] + 0.75 * c2[0, t, h][:, None] * S20[0, h]
            np.testing.assert_allclose(o[0, t, h], q[0, t, h] @ mix, rtol=1e-12, atol=1e-13)


def test_batch_head_independence_and_permutation():
    q, k, v, g1, g2 = rand_case(800, B=3, H=4)
    gam = np.array([0.1, 0.4, 0.7, 0.95])
    o, S1, S2 = orc.recurrent(q, k, v, g1, g2, gam)
    pb, ph = [2, 0, 1], [3, 1, 0, 2]

    def perm(x):
        return x[pb][:, :, ph]
    op, S1p, _ = orc.recurrent(perm(q), perm(k), perm(v), perm(g1), perm(g2), gam[ph])
    np.testing.assert_array_equal(op, perm(o))
    np.testing.assert_array_equal(S1p, S1[pb][:, ph])
    # one (b, h) on its own gives the same numbers
    b, h = 1, 2
    o1, s1, _ = orc.recurrent(q[b:b + 1, :, h:h + 1], k[b:b + 1, :, h:h + 1], v[b:b + 1, :, h:h + 1],
                              g1[b:b + 1, :, h:h + 1], g2[b:b + 1, :, h:h + 1], gam[h])
    np.testing.assert_array_equal(o1[0, :, 0], o[b, :, h])
    np.testing.assert_array_equal(s1[0, 0], S1[b, h])


def test_planted_mistakes_are_caught():
    """The pins above would notice the usual slips: emulate each slip in numpy and check
    that it differs from the oracle on the data of a pin."""
    q, k, v, g1, g2 = rand_case(900, B=1, T=8, H=1, dk=3, dv=2, strong=True)
    o, _, _ = orc.recurrent(q, k, v, g1, g2, 0.3)

    def emulate(read_before_update=False, swap_gates=False, decay_current=False):
        S1 = np.zeros((3, 2))
        S2 = np.zeros((3, 2))
        out = []
        for t in range(8):
            a1, a2 = np.exp(g1[0, t, 0]), np.exp(g2[0, t, 0])
            if swap_gates:
                a1, a2 = a2, a1
            kv = np.outer(k[0, t, 0], v[0, t, 0])
            if read_before_update:
                out.append(q[0, t, 0] @ (0.3 * S1 + 0.7 * S2))
            if decay_current:
                S1, S2 = a1[:, None] * (S1 + kv), a2[:, None] * (S2 + kv)
            else:
                S1, S2 = a1[:, None] * S1 + kv, a2[:, None] * S2 + kv
            if not read_before_update:
                out.append(q[0, t, 0] @ (0.3 * S1 + 0.7 * S2))
        return np.array(out)
    np.testing.assert_allclose(emulate(), o[0, :, 0], rtol=1e-12, atol=1e-13)
    for kw in (dict(read_before_update=True), dict(swap_gates=True), dict(decay_current=True)):
        assert np.max(np.abs(emulate(**kw) - o[0, :, 0])) > 1e-3


def test_gate_map_against_sigmoid_power_and_asymptotes():
    """The pre-activation -> log-gate map: alpha = sigmoid(z)^(1/tau), pinned by the direct sigmoid power on a
    moderate range, by its values at 0, by both asymptotes, by sigmoid's reflection identity at tau = 1 and by
    its derivative sigmoid(-z) / tau (a sign error, a missing 1/tau or softplus(+z) fails several of these)."""
    import math
    z = np.linspace(-12.0, 12.0, 97)
    for tau in (1.0, 4.0, 16.0):
        g = orc.log_gates_from_preactivations(z, tau)
        assert g.dtype == np.float64 and np.all(g < 0)
        direct = (1.0 / (1.0 + np.exp(-z))) ** (1.0 / tau)
        np.testing.assert_allclose(np.exp(g), direct, rtol=1e-13)
        assert abs(float(orc.log_gates_from_preactivations(0.0, tau)) + math.log(2.0) / tau) < 1e-16
        assert np.all(np.diff(g) > 0)                       # more positive z = less forgetting
        # z -> -inf: alpha -> e^(z/tau);  z -> +inf: log alpha -> -e^-z / tau (no overflow, no flush to zero)
        assert abs(float(orc.log_gates_from_preactivations(-60.0, tau)) + 60.0 / tau) < 1e-20
        assert float(orc.log_gates_from_preactivations(-800.0, tau)) == -800.0 / tau
        hi = float(orc.log_gates_from_preactivations(40.0, tau))
        assert hi < 0 and abs(hi * tau / -math.exp(-40.0) - 1.0) < 1e-12
        # derivative by central differences
        h = 1e-5
        num = (orc.log_gates_from_preactivations(z + h, tau) - orc.log_gates_from_preactivations(z - h, tau)) / (2 * h)
        np.testing.assert_allclose(num, (1.0 / (1.0 + np.exp(z))) / tau, rtol=1e-8, atol=1e-12)
    g = orc.log_gates_from_preactivations(z, 1.0)
    np.testing.assert_allclose(np.exp(g) + np.exp(g[::-1]), 1.0, rtol=1e-14)   # sigmoid(z) + sigmoid(-z) = 1


def test_attention_entropy_pins():
    """Entropy of the final query's attention row: uniform scores give log T, one dominant key gives the two-level
    closed form, a shift of all scores changes nothing, keys scaled by c behave like scale scaled by c, and a
    brute-force loop over a tiny case agrees (a missing minus sign, log of the scores instead of the weights, or a
    softmax over the wrong axis fails at least one)."""
    import math
    from oracle import attention as ent
    rng = np.random.default_rng(3)
    B, T, H, d = 2, 37, 3, 8
    k = rng.standard_normal((B, T, H, d))
    q = rng.standard_normal((B, H, d))
    # uniform: q = 0 -> every score 0 -> H = log T
    np.testing.assert_allclose(ent.attention_entropy(np.zeros_like(q), k, 1.0), math.log(T), rtol=1e-14)
    # keys all equal -> uniform as well, whatever q is
    np.testing.assert_allclose(ent.attention_entropy(q, np.broadcast_to(k[:, :1], k.shape), 0.7), math.log(T), rtol=1e-12)
    # two-level scores: key 5 scores c, all others 0:  p = e^c / (e^c + T - 1) on it, (1 - p) / (T - 1) on each other
    kk = np.zeros((1, T, 1, d)); kk[0, 5, 0, 0] = 1.0
    qq = np.zeros((1, 1, d)); qq[0, 0, 0] = 3.0
    c = 3.0 * 0.5
    p = math.exp(c) / (math.exp(c) + T - 1)
    want = -(p * math.log(p) + (1 - p) * math.log((1 - p) / (T - 1)))
    np.testing.assert_allclose(ent.attention_entropy(qq, kk, 0.5), want, rtol=1e-13)
    # a dominant key: entropy -> 0 from above; no NaN from 0 log 0
    qq[0, 0, 0] = 2000.0
    h0 = ent.attention_entropy(qq, kk, 1.0)
    assert h0.shape == (1, 1) and 0.0 <= h0[0, 0] < 1e-300
    # shift invariance: adding the same vector u to every key adds q.u to every score
    base = ent.attention_entropy(q, k, 0.3)
    u = rng.standard_normal((B, 1, H, d))
    np.testing.assert_allclose(ent.attention_entropy(q, k + u, 0.3), base, rtol=1e-10)
    np.testing.assert_allclose(ent.attention_entropy(q, 2.0 * k, 0.15), base, rtol=1e-12)
    assert np.all(base > 0) and np.all(base < math.log(T))
    # brute force
    for b in range(B):
        for h in range(H):
            s = [0.3 * sum(q[b, h, j] * k[b, t, h, j] for j in range(d)) for t in range(T)]
            z = sum(math.exp(x) for x in s)
            hb = -sum(math.exp(x) / z * math.log(math.exp(x) / z) for x in s)
            assert abs(hb - base[b, h]) < 1e-12
    # permutation of the keys changes nothing; heads and batches are independent
    perm = rng.permutation(T)
    np.testing.assert_allclose(ent.attention_entropy(q, k[:, perm], 0.3), base, rtol=1e-12)
    np.testing.assert_allclose(ent.attention_entropy(q[1:], k[1:], 0.3), base[1:], rtol=1e-14)


def test_attention_decode_pins():
    """Single-query softmax attention: q = 0 gives the mean of the values, a dominant key returns its value, the
    output is linear in v and a convex combination of the values, a two-key case has a closed form, and a brute-force
    loop agrees (a missing normaliser, a softmax over features, or k and v swapped fails at least one)."""
    import math
    from oracle import attention as ent
    rng = np.random.default_rng(4)
    B, T, H, d = 2, 29, 3, 8
    k = rng.standard_normal((B, T, H, d))
    v = rng.standard_normal((B, T, H, d))
    q = rng.standard_normal((B, H, d))
    np.testing.assert_allclose(ent.attention_decode(np.zeros_like(q), k, v, 1.0), v.mean(axis=1), rtol=1e-13, atol=1e-15)
    # dominant key 7
    kk = np.zeros_like(k); kk[:, 7] = 50.0 * q / np.sum(q * q, axis=-1, keepdims=True)
    np.testing.assert_allclose(ent.attention_decode(q, kk, v, 1.0), v[:, 7], rtol=1e-12, atol=1e-12)
    base = ent.attention_decode(q, k, v, 0.4)
    # linear in v; convex combination: within the range of the values, per feature
    v2 = rng.standard_normal(v.shape)
    np.testing.assert_allclose(ent.attention_decode(q, k, 2.0 * v - 3.0 * v2, 0.4),
                               2.0 * base - 3.0 * ent.attention_decode(q, k, v2, 0.4), rtol=1e-11, atol=1e-12)
    assert np.all(base <= v.max(axis=1) + 1e-12) and np.all(base >= v.min(axis=1) - 1e-12)
    # two keys: weights sigmoid(+-(s0 - s1))
    q2 = np.array([[[1.0, 2.0]]]); k2 = np.array([[[[0.5, -1.0]], [[2.0, 0.25]]]]); v2k = np.array([[[[1.0, 0.0]], [[0.0, 1.0]]]])
    s0, s1 = 0.3 * (0.5 - 2.0), 0.3 * (2.0 + 0.5)
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    np.testing.assert_allclose(ent.attention_decode(q2, k2, v2k, 0.3)[0, 0], [w0, 1.0 - w0], rtol=1e-14)
    # brute force
    for b in range(B):
        for h in range(H):
            s = [0.4 * sum(q[b, h, j] * k[b, t, h, j] for j in range(d)) for t in range(T)]
            z = sum(math.exp(x) for x in s)
            for j in range(d):
                o = sum(math.exp(s[t]) / z * v[b, t, h, j] for t in range(T))
                assert abs(o - base[b, h, j]) < 1e-12
    # the weights behind it are the ones whose entropy the other function returns: with one-hot values
    # v_i = e_i the output IS the attention row
    Tn = 6
    eye = np.zeros((1, Tn, 1, Tn)); eye[0, :, 0, :] = np.eye(Tn)
    kq = rng.standard_normal((1, Tn, 1, 4)); qq = rng.standard_normal((1, 1, 4))
    a = ent.attention_decode(qq, kq, eye, 0.7)[0, 0]
    assert abs(a.sum() - 1.0) < 1e-14
    assert abs(-np.sum(a * np.log(a)) - ent.attention_entropy(qq, kq, 0.7)[0, 0]) < 1e-13


# ---------------------------------------------------------------- N states, outer-product gate, grouped heads
def nstate_case(seed, N=3, B=2, T=11, H=4, Hkv=2, dk=5, dv=4, beta=True):
    q = rnd(seed, B, T, H, dk)
    k, v = rnd(seed + 1, B, T, Hkv, dk), rnd(seed + 2, B, T, Hkv, dv)
    ga = -np.random.default_rng(seed + 3).uniform(0.0, 1.0, (N, B, T, H, dk))
    gb = -np.random.default_rng(seed + 4).uniform(0.0, 0.7, (N, B, T, H, dv)) if beta else None
    w = np.random.default_rng(seed + 5).uniform(-0.5, 1.0, (N, H))
    S0 = rnd(seed + 6, N, B, H, dk, dv)
    return q, k, v, ga, gb, w, S0


def test_nstate_hand_example_outer_gate():
    rows = np.loadtxt(os.path.join(GOLD, "hand_example_outer_gate.txt"))
    T = rows.shape[0]
    one = np.ones((1, T, 1, 1))
    ga = np.log(np.array([0.5, 1.0])).reshape(2, 1, 1, 1, 1) * np.ones((2, 1, T, 1, 1))
    gb = np.log(np.array([0.5, 0.5])).reshape(2, 1, 1, 1, 1) * np.ones((2, 1, T, 1, 1))
    o, S = orc.nstate(one, one, one, ga, gb, [0.25, 0.75])
    np.testing.assert_allclose(o.ravel(), rows[:, 3], atol=1e-15)
    for t in range(T):
        _, St = orc.nstate(one[:, :t + 1], one[:, :t + 1], one[:, :t + 1], ga[:, :, :t + 1], gb[:, :, :t + 1], [0.25, 0.75])
        assert St[0].ravel()[0] == pytest.approx(rows[t, 1], abs=1e-15)
        assert St[1].ravel()[0] == pytest.approx(rows[t, 2], abs=1e-15)


def test_nstate_reduces_to_the_dual_state_recurrence_bit_for_bit():
    q, k, v, g1, g2 = rand_case(500, B=2, T=17, H=3, dk=6, dv=5)
    S1, S2 = rnd(501, 2, 3, 6, 5), rnd(502, 2, 3, 6, 5)
    gamma, scale = 0.3, 0.8
    ro, rS1, rS2 = orc.recurrent(q, k, v, g1, g2, gamma, scale, S1=S1, S2=S2)
    for gb in (None, np.zeros((2, 2, 17, 3, 5))):      # no beta gate, and beta = 1 given explicitly
        o, S = orc.nstate(q, k, v, np.stack([g1, g2]), gb, [gamma, 1.0 - gamma], scale, S=np.stack([S1, S2]))
        assert np.array_equal(o, ro) and np.array_equal(S[0], rS1) and np.array_equal(S[1], rS2)
    # one state = the dual-state layer with the second state switched off
    o1, S = orc.nstate(q, k, v, g1[None], None, [1.0], scale, S=S1[None])
    ro1, rS1b, _ = orc.recurrent(q, k, v, g1, g2, 1.0, scale, S1=S1, S2=S2)
    np.testing.assert_allclose(o1, ro1, rtol=0, atol=1e-13)
    assert np.array_equal(S[0], rS1b)


def test_nstate_brute_force_python_loops():
    N, B, T, H, Hkv, dk, dv = 3, 1, 6, 4, 2, 3, 2
    q, k, v, ga, gb, w, S0 = nstate_case(520, N, B, T, H, Hkv, dk, dv)
    o, S = orc.nstate(q, k, v, ga, gb, w, 0.7, S=S0)
    ref_o = np.zeros((B, T, H, dv))
    ref_S = S0.copy()
    for b in range(B):
        for h in range(H):
            hk = h // (H // Hkv)
            for t in range(T):
                for n in range(N):
                    for d in range(dk):
                        for j in range(dv):
                            ref_S[n, b, h, d, j] = (np.exp(ga[n, b, t, h, d]) * np.exp(gb[n, b, t, h, j]) * ref_S[n, b, h, d, j]
                                                    + k[b, t, hk, d] * v[b, t, hk, j])
                for j in range(dv):
                    ref_o[b, t, h, j] = 0.7 * sum(q[b, t, h, d] * sum(w[n, h] * ref_S[n, b, h, d, j] for n in range(N))
                                                  for d in range(dk))
    np.testing.assert_allclose(o, ref_o, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, ref_S, rtol=1e-13, atol=1e-13)


def test_nstate_unrolled_form_with_both_gate_vectors():
    """Zero initial states: o_t[j] = scale sum_n w_n sum_{s<=t} (sum_d q_t[d] k_s[d] A^n_ts[d]) B^n_ts[j] v_s[j], with A and B
    the products of alpha and beta over tau = s+1 .. t, taken here from cumulative sums of the log-gates."""
    N, B, T, H, Hkv, dk, dv = 2, 1, 9, 2, 1, 4, 3
    q, k, v, ga, gb, w, _ = nstate_case(530, N, B, T, H, Hkv, dk, dv)
    o, _ = orc.nstate(q, k, v, ga, gb, w, 1.3)
    ca, cb = np.cumsum(ga, axis=2), np.cumsum(gb, axis=2)
    ref = np.zeros_like(o)
    for h in range(H):
        for t in range(T):
            for s_ in range(t + 1):
                for n in range(N):
                    A = np.exp(ca[n, 0, t, h] - ca[n, 0, s_, h])
                    Bv = np.exp(cb[n, 0, t, h] - cb[n, 0, s_, h])
                    ref[0, t, h] += 1.3 * w[n, h] * np.sum(q[0, t, h] * k[0, s_, 0] * A) * Bv * v[0, s_, 0]
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-12)


def test_nstate_geometric_closed_form_and_linearity_in_the_blend():
    N, T, dk, dv = 2, 40, 3, 2
    a = np.array([[0.9, 0.5, 1.0], [0.7, 0.99, 0.2]])
    bt = np.array([[0.8, 1.0], [0.6, 0.95]])
    kk, vv = np.array([0.3, -1.2, 2.0]), np.array([1.5, -0.4])
    ga = np.log(a).reshape(N, 1, 1, 1, dk) * np.ones((N, 1, T, 1, dk))
    gb = np.log(bt).reshape(N, 1, 1, 1, dv) * np.ones((N, 1, T, 1, dv))
    k = kk.reshape(1, 1, 1, dk) * np.ones((1, T, 1, dk))
    v = vv.reshape(1, 1, 1, dv) * np.ones((1, T, 1, dv))
    q = rnd(541, 1, T, 1, dk)
    o, S = orc.nstate(q, k, v, ga, gb, [0.4, 0.6])
    for n in range(N):
        r = a[n][:, None] * bt[n][None, :]
        geo = np.where(r == 1.0, float(T), (1.0 - r ** T) / np.where(r == 1.0, 1.0, 1.0 - r))
        np.testing.assert_allclose(S[n, 0, 0], geo * np.outer(kk, vv), rtol=1e-12)
    parts = [orc.nstate(q, k, v, ga, gb, e)[0] for e in ([1.0, 0.0], [0.0, 1.0])]
    np.testing.assert_allclose(o, 0.4 * parts[0] + 0.6 * parts[1], rtol=1e-12, atol=1e-13)


def test_nstate_grouped_heads_equal_repeated_heads_and_planted_mistakes():
    N, B, T, H, Hkv, dk, dv = 4, 2, 7, 6, 2, 4, 4
    q, k, v, ga, gb, w, S0 = nstate_case(550, N, B, T, H, Hkv, dk, dv)
    o, S = orc.nstate(q, k, v, ga, gb, w, 1.0, S=S0)
    o_rep, S_rep = orc.nstate(q, np.repeat(k, H // Hkv, axis=2), np.repeat(v, H // Hkv, axis=2), ga, gb, w, 1.0, S=S0)
    assert np.array_equal(o, o_rep) and np.array_equal(S, S_rep)
    # mistakes that must show: heads interleaved instead of grouped, beta taken for alpha, states swapped in the blend
    o_bad, _ = orc.nstate(q, np.tile(k, (1, 1, H // Hkv, 1)), np.tile(v, (1, 1, H // Hkv, 1)), ga, gb, w, 1.0, S=S0)
    assert np.max(np.abs(o_bad - o)) > 1e-3
    o_bad, _ = orc.nstate(q, k, v, gb, ga, w, 1.0, S=S0)          # dk == dv here, so the swap is well formed
    assert np.max(np.abs(o_bad - o)) > 1e-3
    o_bad, _ = orc.nstate(q, k, v, ga, gb, w[::-1].copy(), 1.0, S=S0)
    assert np.max(np.abs(o_bad - o)) > 1e-3


def test_attention_prefill_pins():
    """Causal softmax attention over a prompt: the first position returns v_0; zero queries give the running mean of
    the values; every row equals the single-query oracle on the prefix it may see; a brute-force loop."""
    from oracle import attention as att
    B, T, H, d = 2, 19, 3, 8
    q, k, v = rnd(700, B, T, H, d), rnd(701, B, T, H, d), rnd(702, B, T, H, d)
    o = att.attention_prefill(q, k, v, 0.6)
    np.testing.assert_allclose(o[:, 0], v[:, 0], rtol=1e-14)
    o0 = att.attention_prefill(np.zeros_like(q), k, v, 0.6)
    np.testing.assert_allclose(o0, np.cumsum(v, axis=1) / np.arange(1, T + 1).reshape(1, T, 1, 1), rtol=1e-12)
    for t in (0, 5, T - 1):
        np.testing.assert_allclose(o[:, t], att.attention_decode(q[:, t], k[:, :t + 1], v[:, :t + 1], 0.6), rtol=1e-12)
    ref = np.zeros_like(o)
    for b in range(B):
        for h in range(H):
            for t in range(T):
                w = [np.exp(0.6 * float(np.dot(q[b, t, h], k[b, i, h]))) for i in range(t + 1)]
                ref[b, t, h] = sum(wi * v[b, i, h] for i, wi in enumerate(w)) / sum(w)
    np.testing.assert_allclose(o, ref, rtol=1e-11)
    # a key far ahead of the query must not matter: changing the future leaves the past untouched
    k2, v2 = k.copy(), v.copy()
    k2[:, 10:] += 3.0
    v2[:, 10:] -= 5.0
    np.testing.assert_array_equal(att.attention_prefill(q, k2, v2, 0.6)[:, :10], o[:, :10])


def test_controller_oracle_pins():
    """The conversion logic against the paper's own table and hand-worked cases."""
    from oracle import controller as ctl
    table = np.loadtxt(os.path.join(GOLD, "conversion_rate_table.txt"))
    for lo, hi, pct in table:
        hi = int(hi) if hi > 0 else 1 << 20
        for L in (int(lo), (int(lo) + hi) // 2, hi - 1):
            assert ctl.max_conversion_rate(L) == pct / 100.0, L
    # the rates of the table on a 32-layer model: 4, 8, 12 and 16 layers
    assert [int(ctl.max_conversion_rate(L) * 32) for L in (100, 3000, 5000, 20000)] == [4, 8, 12, 16]
    sens = [0.7, 0.2, 0.9, 0.2, 0.05]
    assert ctl.rank_layers(sens) == list(np.argsort(np.array(sens), kind="stable")) == [4, 1, 3, 0, 2]
    # Section 5.3 formula by hand: Llama-2-7B (32 layers, 32 heads of 128) in bf16 at 4096 tokens: 16 KiB per token and
    # layer, 64 MiB per layer, 2 GiB for the model
    assert ctl.kv_cache_bytes(1, 1, 1, 32, 128, 2) == 16384
    assert ctl.kv_cache_bytes(32, 1, 4096, 32, 128, 2) == 2 * 1024 ** 3
    order = [3, 1, 0, 2]
    # each conversion frees 12 - 2 = 10: 100 -> 90 -> 80 -> 70
    assert ctl.conversion_plan(order, 100, 70, 12, 2, 1.0) == ([3, 1, 0], 70, "memory relief")
    assert ctl.conversion_plan(order, 100, 70, 12, 2, 0.5) == ([3, 1], 80, "quality limit")
    assert ctl.conversion_plan(order, 60, 70, 12, 2, 1.0) == ([], 60, "no pressure")
    assert ctl.conversion_plan(order, 100, 10, 12, 2, 1.0) == ([3, 1, 0, 2], 60, "all converted")
    assert ctl.conversion_plan(order, 100, 99, 12, 2, 0.125) == ([], 100, "quality limit")   # 12.5 % of 4 layers: none


def test_oracle_threads_reported():
    assert orc.threads() >= 1
