"""ctypes front end of the C oracle (oracle/dsla_oracle.c).

Test infrastructure only.  Inputs are numpy arrays of any float dtype; they are
widened to fp64 exactly and every result is fp64.

Layouts follow the layer statement of Section 4.1 of the paper:
  q, k, g1, g2 : [B, T, H, dk]   (g = natural log of the forget gate, <= 0)
  v, o         : [B, T, H, dv]
  S1, S2       : [B, H, dk, dv]  (history, recency)
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ci = ctypes.c_int
        lib.dsla_oracle_recurrent.argtypes = [ci] * 5 + [dp] * 6 + [ctypes.c_double, dp, dp, dp]
        lib.dsla_oracle_recurrent.restype = None
        lib.dsla_oracle_unrolled.argtypes = [ci] * 5 + [dp] * 6 + [ctypes.c_double, dp]
        lib.dsla_oracle_unrolled.restype = None
        lib.dsla_oracle_nstate.argtypes = [ci] * 7 + [dp] * 6 + [ctypes.c_double, dp, dp]
        lib.dsla_oracle_nstate.restype = None
        lib.dsla_oracle_threads.argtypes = []
        lib.dsla_oracle_threads.restype = ci
        _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads the oracle's (batch, head) loop uses."""
    return int(_load().dsla_oracle_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _gamma_vec(gamma, H):
    g = np.asarray(gamma, dtype=np.float64)
    if g.ndim == 0:
        g = np.full((H,), float(g), dtype=np.float64)
    assert g.shape == (H,)
    return np.ascontiguousarray(g)


def log_gates_from_preactivations(z, tau):
    """log alpha for alpha = sigmoid(z) ** (1 / tau), fp64.

    The paper does not print the map from the gate projections to (0,1] (Section 4.1 calls the gates
    data-driven, Section 5.3 says they come from single linear layers); this is the reading taken: the
    temperature-sigmoid of the gated linear attention work the method extends.  Written from the definition,
    log alpha = -log(1 + e^-z) / tau, with the library's overflow-free log-sum-exp for the logarithm.
    """
    z = np.asarray(z, dtype=np.float64)
    assert float(tau) > 0.0
    return -np.logaddexp(0.0, -z) / float(tau)


def recurrent(q, k, v, g1, g2, gamma, scale=1.0, S1=None, S2=None):
    """Token-by-token DSLA recurrence (Section 4.1, state-update and read-out equations).

    Returns (o, S1_final, S2_final), all fp64.  S1/S2 default to zeros; when given
    they are the carried-in states and are not modified (copies are returned).
    A decode step is the call with T == 1.
    """
    q, k, v, g1, g2 = map(_f64, (q, k, v, g1, g2))
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (B, T, H, dk) and g1.shape == (B, T, H, dk) and g2.shape == (B, T, H, dk)
    assert v.shape == (B, T, H, dv)
    gm = _gamma_vec(gamma, H)
    S1 = np.zeros((B, H, dk, dv)) if S1 is None else _f64(S1).copy()
    S2 = np.zeros((B, H, dk, dv)) if S2 is None else _f64(S2).copy()
    assert S1.shape == (B, H, dk, dv) and S2.shape == (B, H, dk, dv)
    o = np.zeros((B, T, H, dv), dtype=np.float64)
    _load().dsla_oracle_recurrent(B, T, H, dk, dv, _ptr(q), _ptr(k), _ptr(v), _ptr(g1), _ptr(g2),
                                  _ptr(gm), float(scale), _ptr(S1), _ptr(S2), _ptr(o))
    return o, S1, S2


def unrolled(q, k, v, g1, g2, gamma, scale=1.0):
    """O(T^2) attention-score form with zero initial states (Section 4.1, last display,
    applied to every query position).  Returns o (fp64)."""
    q, k, v, g1, g2 = map(_f64, (q, k, v, g1, g2))
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gm = _gamma_vec(gamma, H)
    o = np.zeros((B, T, H, dv), dtype=np.float64)
    _load().dsla_oracle_unrolled(B, T, H, dk, dv, _ptr(q), _ptr(k), _ptr(v), _ptr(g1), _ptr(g2),
                                 _ptr(gm), float(scale), _ptr(o))
    return o


def nstate(q, k, v, galpha, gbeta=None, w=None, scale=1.0, S=None):
    """The recurrence with N states, outer-product gates alpha^T beta and grouped key/value heads
    (oracle/dsla_oracle.c: dsla_oracle_nstate; background section on gated linear attention, Section 4.2,
    the ablation over the number of states in Section 5.5).

    q [B,T,H,dk]; k [B,T,Hkv,dk]; v [B,T,Hkv,dv]; galpha [N,B,T,H,dk] = log alpha; gbeta [N,B,T,H,dv] = log beta or
    None (beta = 1); w [N] or [N,H] blend coefficients (default: 1/N each); S [N,B,H,dk,dv] initial states or None
    (zeros).  Returns (o [B,T,H,dv], S_final [N,B,H,dk,dv]), fp64.
    """
    q, k, v, galpha = map(_f64, (q, k, v, galpha))
    N, B, T, H, dk = galpha.shape
    Hkv, dv = v.shape[2], v.shape[3]
    assert q.shape == (B, T, H, dk) and k.shape == (B, T, Hkv, dk) and v.shape == (B, T, Hkv, dv)
    assert H % Hkv == 0
    gb = None
    if gbeta is not None:
        gb = _f64(gbeta)
        assert gb.shape == (N, B, T, H, dv)
    wv = np.full((N, H), 1.0 / N) if w is None else np.asarray(w, dtype=np.float64)
    if wv.ndim == 1:
        wv = np.repeat(wv[:, None], H, axis=1)
    wv = np.ascontiguousarray(wv)
    assert wv.shape == (N, H)
    S = np.zeros((N, B, H, dk, dv)) if S is None else _f64(S).copy()
    assert S.shape == (N, B, H, dk, dv)
    o = np.zeros((B, T, H, dv))
    _load().dsla_oracle_nstate(N, B, T, H, Hkv, dk, dv, _ptr(q), _ptr(k), _ptr(v), _ptr(galpha),
                               _ptr(gb) if gb is not None else None, _ptr(wv), float(scale), _ptr(S), _ptr(o))
    return o, S
