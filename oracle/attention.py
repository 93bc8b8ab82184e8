"""CPU oracle of the two softmax-attention pieces beside the DSLA layer: the attention-entropy sensitivity signal and
the single-query (decode) attention of an unconverted layer.  TEST INFRASTRUCTURE: only tests/, the smoke check and
the benchmark's CPU baseline may import this; the product path never does.

What it computes (Section 4.3, "Layer Ranking via Sensitivity"): for the final query q_T of a softmax-attention
head, the attention distribution over the keys, A_i = softmax_i(scale * q_T . k_i), i = 0..T-1, and its Shannon
entropy.  The paper's display prints sum_i A_i log A_i without a minus sign while the text around it takes a low
value to mean attention concentrated on few tokens; the reading taken is the entropy proper, H = -sum_i A_i log A_i >= 0
(natural logarithm), which is the negative of the printed sum.  Plain numpy, fp64, one (batch, head) at a time
through library primitives (matrix-vector product, exp, log, sum); no blocking or streaming.
"""
import numpy as np


def attention_entropy(q_last, k, scale):
    """q_last: [B, H, d]; k: [B, T, H, d]; returns H: [B, H] fp64.  A term with A_i == 0 contributes 0."""
    q_last = np.asarray(q_last, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, T, H, d = k.shape
    assert q_last.shape == (B, H, d) and T >= 1
    out = np.zeros((B, H), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            s = float(scale) * (k[b, :, h, :] @ q_last[b, h])      # scores of the final query against every key
            e = np.exp(s - s.max())
            a = e / e.sum()                                         # the attention row
            nz = a > 0
            out[b, h] = -np.sum(a[nz] * np.log(a[nz]))
    return out


def attention_decode(q_last, k, v, scale):
    """Softmax attention of one query per (batch, head) over T cached keys and values: the decode step of a layer
    that has NOT been converted, which the paper's serving system runs beside the DSLA layers (Section 4.3; its
    cost grows with the context, Section 5.3).  o = sum_i softmax_i(scale * q . k_i) v_i, fp64, from the definition.
    q_last: [B, H, d]; k, v: [B, T, H, d]; returns o: [B, H, d]."""
    q_last = np.asarray(q_last, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, T, H, d = k.shape
    assert q_last.shape == (B, H, d) and v.shape[:3] == (B, T, H) and T >= 1
    out = np.zeros((B, H, v.shape[3]), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            s = float(scale) * (k[b, :, h, :] @ q_last[b, h])
            e = np.exp(s - s.max())
            a = e / e.sum()
            out[b, h] = a @ v[b, :, h, :]
    return out


def attention_prefill(q, k, v, scale):
    """Causal softmax attention of a layer that has NOT been converted, over a whole prompt (the Transformer path
    the paper measures the converted layers against, Section 5.3): for every query position t,
    o_t = sum_{i <= t} softmax_{i <= t}(scale * q_t . k_i) v_i.  fp64, from the definition: the full score matrix of
    one (batch, head) through library primitives (matmul, exp, sum), positions after the query set to -inf.
    q, k: [B, T, H, d]; v: [B, T, H, dv]; returns o: [B, T, H, dv]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, T, H, d = q.shape
    assert k.shape == (B, T, H, d) and v.shape[:3] == (B, T, H)
    out = np.zeros((B, T, H, v.shape[3]), dtype=np.float64)
    future = np.triu(np.ones((T, T), dtype=bool), 1)
    for b in range(B):
        for h in range(H):
            s = float(scale) * (q[b, :, h, :] @ k[b, :, h, :].T)
            s[future] = -np.inf
            e = np.exp(s - s.max(axis=1, keepdims=True))
            out[b, :, h, :] = (e / e.sum(axis=1, keepdims=True)) @ v[b, :, h, :]
    return out
