"""Seeded synthetic inputs for the DSLA layer (shared by tests, smoke and bench).

Holds no arithmetic of the method itself: only random draws, the rounding of the
draws to the storage dtype, and the map from gate pre-activations to log-gates that
defines the value distribution of the workload.  numpy only.

Recipe (stands in for Llama-2-7B attention activations, which are not available):
  q, k, v          ~ N(0, 1) * qk_scale                      [B, T, H, d]
  gate pre-act. z  ~ N(2, 1), independent draws for the history and recency gate
  log-gate         g = -softplus(-z) / tau   (= log(sigmoid(z)**(1/tau)) <= 0)
  seed of tensor j of a workload = base_seed + j
All tensors are returned as float32 arrays whose values are exactly representable
in the requested storage dtype (bf16 values are rounded to nearest even first).
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20250609


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def log_gate_from_preact(z: np.ndarray, tau: float) -> np.ndarray:
    """g = log(sigmoid(z) ** (1 / tau)) = -softplus(-z) / tau, computed in fp64."""
    z = np.asarray(z, dtype=np.float64)
    return (-np.logaddexp(0.0, -z) / float(tau)).astype(np.float32)


def layer_inputs(seed: int, B: int, T: int, H: int, dk: int, dv: int, *, io_dtype: str = "bf16",
                 gate_dtype: str = "f32", tau: float = 16.0, qk_scale: float = 1.0,
                 gate_mean: float = 2.0, gates: str = "log") -> dict:
    """One batch of layer inputs: dict with q, k, g1, g2 [B,T,H,dk] and v [B,T,H,dv].
    gates = "log": g1, g2 are log-gates; "preact": they are the pre-activations z themselves (same draws)."""
    assert gates in ("log", "preact")
    out = {}
    for j, (name, d) in enumerate((("q", dk), ("k", dk), ("v", dv))):
        rng = np.random.default_rng(seed + j)
        x = rng.standard_normal((B, T, H, d), dtype=np.float32) * np.float32(qk_scale)
        out[name] = _store(x, io_dtype)
    for j, name in enumerate(("g1", "g2")):
        rng = np.random.default_rng(seed + 3 + j)
        z = rng.standard_normal((B, T, H, dk), dtype=np.float32) + np.float32(gate_mean)
        out[name] = _store(z if gates == "preact" else log_gate_from_preact(z, tau), gate_dtype)
    return out


def initial_states(seed: int, B: int, H: int, dk: int, dv: int, amplitude: float = 1.0):
    """Non-zero fp32 states, for tests of carried-in state."""
    r1 = np.random.default_rng(seed + 11)
    r2 = np.random.default_rng(seed + 12)
    S1 = r1.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(amplitude)
    S2 = r2.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(amplitude)
    return S1, S2


# The configurations the build is measured on (shapes of a Llama-2-7B attention layer:
# 32 heads of width 128).  "seed" follows base + 1000 * configuration index.
CONFIGS = {
    "cfg1": dict(B=1, T=256, H=4, dk=64, dv=64, chunk=64, io_dtype="f32", gate_dtype="f32",
                 qk_scale=1.0, decode_steps=16, seed=BASE_SEED + 1000),
    "cfg2": dict(B=1, T=4096, H=32, dk=128, dv=128, chunk=64, io_dtype="bf16", gate_dtype="bf16",
                 qk_scale=128 ** -0.5, seed=BASE_SEED + 2000),
    "cfg3_16k": dict(B=1, T=16384, H=32, dk=128, dv=128, chunk=64, io_dtype="bf16",
                     gate_dtype="bf16", qk_scale=128 ** -0.5, seed=BASE_SEED + 3000),
    "cfg3_64k": dict(B=1, T=65536, H=32, dk=128, dv=128, chunk=64, io_dtype="bf16",
                     gate_dtype="bf16", qk_scale=128 ** -0.5, seed=BASE_SEED + 3500),
    "cfg4": dict(B=64, T=2048, H=32, dk=128, dv=128, chunk=64, io_dtype="bf16", gate_dtype="bf16",
                 qk_scale=128 ** -0.5, decode_steps=256, seed=BASE_SEED + 4000),
    # the DSLA layers of a hybrid 32-layer stack: 16 layer instances, each with its own blend coefficient
    # (drawn by the caller from U(0.2, 0.8) with the layer's seed) and its own inputs; seed of layer l = seed + 10 l
    "cfg5": dict(B=8, T=8192, H=32, dk=128, dv=128, chunk=64, io_dtype="bf16", gate_dtype="bf16",
                 qk_scale=128 ** -0.5, decode_steps=128, layers=16, seed=BASE_SEED + 5000),
}
