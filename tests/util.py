"""Helpers shared by the GPU parity tests: numpy <-> torch marshalling, the error norm,
and a runner that pushes one workload through the C-ABI library."""
import numpy as np

import paper_2506_09316_amd as dsla
from paper_2506_09316_amd.binding import DSLA_BF16, DSLA_F32


def max_rel_err(x, ref):
    """max_i |x_i - ref_i| / max_i |ref_i| over one tensor (the norm the tolerances are stated in)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(x - ref)) / (den if den > 0 else 1.0))


def row_rel_err(x, ref, floor=1e-2):
    """The error at the scale of each output row: max over rows (vectors along the last axis) of
    max|x - ref| over the row / max(max|ref| over the row, floor * max|ref| over the tensor).  A quiet row (early
    tokens, a strongly decayed state row) is held to its own magnitude, not to the loudest row of the tensor; rows
    below 1 % of the tensor maximum are held to that 1 %: such a row is small because its terms cancel (the first
    token's output is (q.k) v with a 128-term dot product near zero), and its error is that of the terms."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    top = np.max(np.abs(ref))
    den = np.maximum(np.max(np.abs(ref), axis=-1), floor * (top if top > 0 else 1.0))
    return float(np.max(np.max(np.abs(x - ref), axis=-1) / den))


def elem_rel_err(x, ref, floor=1e-3):
    """Element-wise relative error with a floor: max_i |x_i - ref_i| / max(|ref_i|, floor * max|ref|).
    An element that is small because large terms cancel carries the rounding error of those terms, so in bf16
    this number is not bounded by the operand precision; it is reported, and asserted only in fp32."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    top = np.max(np.abs(ref))
    den = np.maximum(np.abs(ref), floor * (top if top > 0 else 1.0))
    return float(np.max(np.abs(x - ref) / den))


def to_gpu(a, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t


def code(dtype):
    return DSLA_BF16 if dtype == "bf16" else DSLA_F32


class GpuLayer:
    """One DSLA layer instance on the GPU: owns the states and calls the library."""

    def __init__(self, B, H, d, io_dtype, gate_dtype, gamma=0.5, scale=1.0, chunk=0, segments=0,
                 gamma_per_head=None, gate_mode=0, tau=16.0, status=None, zero_init=False, init=True):
        import torch
        self.B, self.H, self.d = B, H, d
        self.io_dtype, self.gate_dtype = io_dtype, gate_dtype
        self.gph = None
        if gamma_per_head is not None:
            self.gph = torch.tensor(np.asarray(gamma_per_head, dtype=np.float32)).cuda()
        self.desc = dsla.make_desc(B, H, d, d, io_dtype=code(io_dtype), gate_dtype=code(gate_dtype), gamma=gamma,
                                   scale=scale, chunk=chunk, segments=segments, gamma_per_head=self.gph,
                                   gate_mode=gate_mode, tau=tau, status=status, zero_init=zero_init)
        self.status = status
        self.S1 = torch.full((B, H, d, d), float("nan"), device="cuda", dtype=torch.float32)
        self.S2 = torch.full((B, H, d, d), float("nan"), device="cuda", dtype=torch.float32)
        if init:   # otherwise the states keep their NaN fill (a zero_init prefill must not read them)
            dsla.dsla_state_init(self.desc, self.S1, self.S2)

    def set_states(self, S1, S2):
        import torch
        self.S1.copy_(torch.from_numpy(np.ascontiguousarray(S1, dtype=np.float32)))
        self.S2.copy_(torch.from_numpy(np.ascontiguousarray(S2, dtype=np.float32)))

    def prefill(self, x):
        import torch
        T = x["q"].shape[1]
        q, k, v = (to_gpu(x[n], self.io_dtype) for n in ("q", "k", "v"))
        g1, g2 = (to_gpu(x[n], self.gate_dtype) for n in ("g1", "g2"))
        o = torch.full_like(v, float("nan"))
        nbytes = dsla.dsla_prefill_workspace_bytes(self.desc, T)
        ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda") if nbytes else None
        dsla.dsla_prefill(self.desc, T, q, k, v, g1, g2, self.S1, self.S2, o, ws)
        torch.cuda.synchronize()
        return o.float().cpu().numpy()

    def decode(self, x):
        """x holds [B, 1, H, d] arrays (one token)."""
        import torch
        q, k, v = (to_gpu(x[n][:, 0], self.io_dtype) for n in ("q", "k", "v"))
        g1, g2 = (to_gpu(x[n][:, 0], self.gate_dtype) for n in ("g1", "g2"))
        o = torch.full_like(v, float("nan"))
        dsla.dsla_decode(self.desc, q, k, v, g1, g2, self.S1, self.S2, o)
        torch.cuda.synchronize()
        return o.float().cpu().numpy()[:, None]

    def states(self):
        return self.S1.cpu().numpy(), self.S2.cpu().numpy()


def slice_t(x, a, b):
    return {n: x[n][:, a:b] for n in x}
