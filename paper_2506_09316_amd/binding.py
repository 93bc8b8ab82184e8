"""ctypes binding of libdsla.so: same entry-point names as include/dsla.h, argument
marshalling only.  Tensors are torch tensors on the GPU; their data pointers and the
current torch HIP stream are handed to the library.  No computation happens here, and
there is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libdsla.so")
_lib = None

DSLA_F32, DSLA_BF16 = 0, 1
KERNEL_NAMES = ("state_init", "prefill_segment_state", "prefill_segment_scan", "prefill_chunk_loop", "decode",
                "prefill_segment_list", "attention_entropy", "attention_decode", "decode_multi", "attention_prefill", "project")
EXPORTS = ("dsla_state_init", "dsla_prefill_workspace_bytes", "dsla_prefill", "dsla_prefill_static_ws", "dsla_decode",
           "dsla_prefill_varlen_workspace_bytes", "dsla_prefill_varlen", "dsla_decode_slots",
           "dsla_decode_multi", "dsla_prefill_multi_workspace_bytes", "dsla_prefill_multi",
           "dsla_attention_entropy_workspace_bytes", "dsla_attention_entropy",
           "dsla_attention_decode_workspace_bytes", "dsla_attention_decode", "dsla_attention_prefill", "dsla_project",
           "dsla_rank_layers", "dsla_max_conversion_rate", "dsla_kv_cache_bytes", "dsla_conversion_plan",
           "dsla_status_string", "dsla_last_hip_error", "dsla_profile_enable", "dsla_profile_collect")


class DslaDesc(ctypes.Structure):
    """Mirror of `dsla_desc` in include/dsla.h."""
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32),
                ("chunk", ctypes.c_int32), ("segments", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("gate_dtype", ctypes.c_int32), ("gate_mode", ctypes.c_int32), ("zero_init", ctypes.c_int32),
                ("tau", ctypes.c_float), ("gamma", ctypes.c_float), ("scale", ctypes.c_float),
                ("gamma_per_head", ctypes.c_void_p), ("status", ctypes.c_void_p)]


class DslaMulti(ctypes.Structure):
    """Mirror of `dsla_multi` in include/dsla.h."""
    _fields_ = [("n_states", ctypes.c_int32), ("H_kv", ctypes.c_int32), ("g_alpha", ctypes.POINTER(ctypes.c_void_p)),
                ("g_beta", ctypes.POINTER(ctypes.c_void_p)), ("S", ctypes.POINTER(ctypes.c_void_p)),
                ("weights", ctypes.POINTER(ctypes.c_float)), ("weights_per_head", ctypes.c_void_p)]


class DslaError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"dsla status {status}: {text}")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libdsla.so (built by paper_2506_09316_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} is not built; run `python -m paper_2506_09316_amd.build` "
                                "(or __graft_entry__.build())")
    # PyTorch ships its own copy of the HIP runtime.  Whichever copy is loaded first serves the whole process, and
    # tensors and kernels must live in the same one: load PyTorch's before the library pulls in the system's.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    vp, dp = ctypes.c_void_p, ctypes.POINTER(DslaDesc)
    lib.dsla_state_init.argtypes = [dp, vp, vp, vp]
    lib.dsla_state_init.restype = ctypes.c_int
    lib.dsla_prefill_workspace_bytes.argtypes = [dp, ctypes.c_int64]
    lib.dsla_prefill_workspace_bytes.restype = ctypes.c_size_t
    lib.dsla_prefill.argtypes = [dp, ctypes.c_int64] + [vp] * 9 + [ctypes.c_size_t, vp]
    lib.dsla_prefill.restype = ctypes.c_int
    lib.dsla_prefill_static_ws.argtypes = [dp, ctypes.c_int64] + [vp] * 9
    lib.dsla_prefill_static_ws.restype = ctypes.c_int
    lib.dsla_decode.argtypes = [dp] + [vp] * 9
    lib.dsla_decode.restype = ctypes.c_int
    lib.dsla_prefill_varlen_workspace_bytes.argtypes = [dp, ctypes.c_int64, ctypes.c_int64]
    lib.dsla_prefill_varlen_workspace_bytes.restype = ctypes.c_size_t
    lib.dsla_prefill_varlen.argtypes = [dp, ctypes.c_int64, ctypes.c_int64] + [vp] * 12 + [ctypes.c_size_t, vp]
    lib.dsla_prefill_varlen.restype = ctypes.c_int
    lib.dsla_decode_slots.argtypes = [dp] + [vp] * 11
    lib.dsla_decode_slots.restype = ctypes.c_int
    mp = ctypes.POINTER(DslaMulti)
    lib.dsla_decode_multi.argtypes = [dp, mp] + [vp] * 5
    lib.dsla_decode_multi.restype = ctypes.c_int
    lib.dsla_prefill_multi_workspace_bytes.argtypes = [dp, mp, ctypes.c_int64]
    lib.dsla_prefill_multi_workspace_bytes.restype = ctypes.c_size_t
    lib.dsla_prefill_multi.argtypes = [dp, mp, ctypes.c_int64] + [vp] * 5 + [ctypes.c_size_t, vp]
    lib.dsla_prefill_multi.restype = ctypes.c_int
    lib.dsla_attention_entropy_workspace_bytes.argtypes = [ctypes.c_int32] * 3 + [ctypes.c_int64]
    lib.dsla_attention_entropy_workspace_bytes.restype = ctypes.c_size_t
    lib.dsla_attention_entropy.argtypes = ([ctypes.c_int32] * 3 + [ctypes.c_int64, ctypes.c_int32, ctypes.c_float]
                                           + [vp] * 4 + [ctypes.c_size_t, vp])
    lib.dsla_attention_entropy.restype = ctypes.c_int
    lib.dsla_attention_decode_workspace_bytes.argtypes = [ctypes.c_int32] * 3 + [ctypes.c_int64]
    lib.dsla_attention_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.dsla_attention_decode.argtypes = ([ctypes.c_int32] * 3 + [ctypes.c_int64, ctypes.c_int32, ctypes.c_float]
                                          + [vp] * 6 + [ctypes.c_size_t, vp])
    lib.dsla_attention_decode.restype = ctypes.c_int
    lib.dsla_project.argtypes = [ctypes.c_int64] + [ctypes.c_int32] * 3 + [vp] * 3 + [ctypes.POINTER(ctypes.c_void_p), vp]
    lib.dsla_project.restype = ctypes.c_int
    lib.dsla_attention_prefill.argtypes = [ctypes.c_int32] * 3 + [ctypes.c_int64, ctypes.c_int32, ctypes.c_float] + [vp] * 5
    lib.dsla_attention_prefill.restype = ctypes.c_int
    lib.dsla_rank_layers.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32)]
    lib.dsla_rank_layers.restype = ctypes.c_int
    lib.dsla_max_conversion_rate.argtypes = [ctypes.c_int64]
    lib.dsla_max_conversion_rate.restype = ctypes.c_float
    lib.dsla_kv_cache_bytes.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64] + [ctypes.c_int32] * 3
    lib.dsla_kv_cache_bytes.restype = ctypes.c_int64
    lib.dsla_conversion_plan.argtypes = ([ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)] + [ctypes.c_int64] * 4
                                         + [ctypes.c_float, ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_int32),
                                            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)])
    lib.dsla_conversion_plan.restype = ctypes.c_int
    lib.dsla_status_string.argtypes = [ctypes.c_int]
    lib.dsla_status_string.restype = ctypes.c_char_p
    lib.dsla_last_hip_error.argtypes = []
    lib.dsla_last_hip_error.restype = ctypes.c_char_p
    lib.dsla_profile_enable.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.dsla_profile_enable.restype = ctypes.c_int
    lib.dsla_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.dsla_profile_collect.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        lib = load_library()
        text = lib.dsla_status_string(status).decode()
        if status == 5:
            text += ": " + lib.dsla_last_hip_error().decode()
        raise DslaError(status, text)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return DSLA_BF16
    if t.dtype == torch.float32:
        return DSLA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous GPU tensors"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_desc(B, H, d_k, d_v, *, io_dtype, gate_dtype, gamma=0.5, scale=1.0, chunk=0, segments=0,
              gamma_per_head=None, gate_mode=0, tau=16.0, zero_init=False, status=None) -> DslaDesc:
    """status: optional int32 GPU tensor of one element (the caller keeps it alive)."""
    gp = ctypes.c_void_p(gamma_per_head.data_ptr()) if gamma_per_head is not None else None
    sp = ctypes.c_void_p(status.data_ptr()) if status is not None else None
    return DslaDesc(int(B), int(H), int(d_k), int(d_v), int(chunk), int(segments), int(io_dtype), int(gate_dtype),
                    int(gate_mode), int(bool(zero_init)), float(tau), float(gamma), float(scale), gp, sp)


def dsla_state_init(desc: DslaDesc, S1, S2):
    """Zero both states (include/dsla.h: dsla_state_init)."""
    _check(load_library().dsla_state_init(ctypes.byref(desc), _ptr(S1), _ptr(S2), _stream()))


def dsla_prefill_workspace_bytes(desc: DslaDesc, T: int) -> int:
    return int(load_library().dsla_prefill_workspace_bytes(ctypes.byref(desc), int(T)))


def dsla_prefill(desc: DslaDesc, T, q, k, v, g1, g2, S1, S2, o, workspace=None):
    """Chunked prefill over T tokens (include/dsla.h: dsla_prefill).  `workspace` is a uint8 GPU
    tensor of at least dsla_prefill_workspace_bytes(desc, T) bytes, or None when that is zero."""
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().dsla_prefill(ctypes.byref(desc), int(T), _ptr(q), _ptr(k), _ptr(v), _ptr(g1), _ptr(g2),
                                       _ptr(S1), _ptr(S2), _ptr(o), _ptr(workspace), wbytes, _stream()))


def dsla_prefill_static_ws(desc: DslaDesc, T, q, k, v, g1, g2, S1, S2, o):
    """dsla_prefill on the library's built-in scratch buffer (include/dsla.h: dsla_prefill_static_ws)."""
    _check(load_library().dsla_prefill_static_ws(ctypes.byref(desc), int(T), _ptr(q), _ptr(k), _ptr(v), _ptr(g1),
                                                 _ptr(g2), _ptr(S1), _ptr(S2), _ptr(o), _stream()))


def dsla_decode(desc: DslaDesc, q, k, v, g1, g2, S1, S2, o):
    """One fused decode step (include/dsla.h: dsla_decode)."""
    _check(load_library().dsla_decode(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g1), _ptr(g2),
                                      _ptr(S1), _ptr(S2), _ptr(o), _stream()))


def dsla_prefill_varlen_workspace_bytes(desc: DslaDesc, total_T: int, max_T: int) -> int:
    return int(load_library().dsla_prefill_varlen_workspace_bytes(ctypes.byref(desc), int(total_T), int(max_T)))


def dsla_prefill_varlen(desc: DslaDesc, total_T, max_T, cu_seqlens, state_slot, q, k, v, g1, g2, S1, S2, o,
                        workspace=None, seq_index=None):
    """Prefill of packed sequences (include/dsla.h: dsla_prefill_varlen).  cu_seqlens: int32 GPU tensor;
    state_slot, seq_index: int32 GPU tensors [B] or None."""
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().dsla_prefill_varlen(ctypes.byref(desc), int(total_T), int(max_T), _ptr(cu_seqlens),
                                              _ptr(seq_index), _ptr(state_slot), _ptr(q), _ptr(k), _ptr(v), _ptr(g1), _ptr(g2),
                                              _ptr(S1), _ptr(S2), _ptr(o), _ptr(workspace), wbytes, _stream()))


def dsla_decode_slots(desc: DslaDesc, q, k, v, g1, g2, state_slot, S1, S2, o, row_index=None):
    """One decode step on states picked from a pool (include/dsla.h: dsla_decode_slots)."""
    _check(load_library().dsla_decode_slots(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(g1), _ptr(g2),
                                            _ptr(row_index), _ptr(state_slot), _ptr(S1), _ptr(S2), _ptr(o), _stream()))


def make_multi(g_alpha, S, weights, *, g_beta=None, H_kv=0, weights_per_head=None) -> DslaMulti:
    """dsla_multi from lists of GPU tensors (one per state).  The returned structure keeps the host arrays it
    points to, and the tensors themselves, alive (attribute _keep)."""
    n = len(g_alpha)
    assert len(S) == n and len(weights) == n and (g_beta is None or len(g_beta) == n)
    ga = (ctypes.c_void_p * n)(*[t.data_ptr() for t in g_alpha])
    gb = None
    if g_beta is not None:
        gb = (ctypes.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in g_beta])
    Sp = (ctypes.c_void_p * n)(*[t.data_ptr() for t in S])
    w = (ctypes.c_float * n)(*[float(x) for x in weights])
    wph = ctypes.c_void_p(weights_per_head.data_ptr()) if weights_per_head is not None else None
    m = DslaMulti(n, int(H_kv), ctypes.cast(ga, ctypes.POINTER(ctypes.c_void_p)),
                  ctypes.cast(gb, ctypes.POINTER(ctypes.c_void_p)) if gb is not None else None,
                  ctypes.cast(Sp, ctypes.POINTER(ctypes.c_void_p)), ctypes.cast(w, ctypes.POINTER(ctypes.c_float)), wph)
    m._keep = (ga, gb, Sp, w, list(g_alpha), list(g_beta) if g_beta is not None else None, list(S), weights_per_head)
    return m


def dsla_decode_multi(desc: DslaDesc, multi: DslaMulti, q, k, v, o):
    """One decode step of a layer with N states (include/dsla.h: dsla_decode_multi)."""
    _check(load_library().dsla_decode_multi(ctypes.byref(desc), ctypes.byref(multi), _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                            _stream()))


def dsla_prefill_multi_workspace_bytes(desc: DslaDesc, multi: DslaMulti, T: int) -> int:
    return int(load_library().dsla_prefill_multi_workspace_bytes(ctypes.byref(desc), ctypes.byref(multi), int(T)))


def dsla_prefill_multi(desc: DslaDesc, multi: DslaMulti, T, q, k, v, o, workspace=None):
    """Prefill of a layer with N states (include/dsla.h: dsla_prefill_multi)."""
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().dsla_prefill_multi(ctypes.byref(desc), ctypes.byref(multi), int(T), _ptr(q), _ptr(k), _ptr(v),
                                             _ptr(o), _ptr(workspace), wbytes, _stream()))


def dsla_attention_entropy_workspace_bytes(B: int, H: int, d: int, T: int) -> int:
    return int(load_library().dsla_attention_entropy_workspace_bytes(int(B), int(H), int(d), int(T)))


def dsla_attention_entropy(q_last, k, entropy, scale: float, workspace=None):
    """Entropy of the final query's attention row (include/dsla.h: dsla_attention_entropy).
    q_last [B,H,d], k [B,T,H,d] (bf16 or fp32 GPU tensors), entropy [B,H] fp32, written."""
    B, T, H, d = k.shape
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().dsla_attention_entropy(int(B), int(H), int(d), int(T), _dtype_code(k), float(scale),
                                                 _ptr(q_last), _ptr(k), _ptr(entropy), _ptr(workspace), wbytes,
                                                 _stream()))


def dsla_attention_decode_workspace_bytes(B: int, H: int, d: int, T: int) -> int:
    return int(load_library().dsla_attention_decode_workspace_bytes(int(B), int(H), int(d), int(T)))


def dsla_attention_decode(q, k, v, o, scale: float, workspace=None, seq_lens=None):
    """Single-query softmax attention over cached keys and values (include/dsla.h: dsla_attention_decode).
    q, o [B,H,d]; k, v [B,T,H,d] (all bf16 or all fp32 GPU tensors); seq_lens: int32 GPU tensor [B] or None."""
    B, T, H, d = k.shape
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().dsla_attention_decode(int(B), int(H), int(d), int(T), _dtype_code(k), float(scale),
                                                _ptr(q), _ptr(k), _ptr(v), _ptr(seq_lens), _ptr(o), _ptr(workspace), wbytes,
                                                _stream()))


def dsla_project(x, W, outs, bias=None):
    """The projections in front of a layer as one GEMM (include/dsla.h: dsla_project).  x [M,K] bf16; W [n_out*width,K]
    bf16; outs: list of n_out bf16 GPU tensors of M*width elements each; bias: fp32 GPU tensor [n_out*width] or None."""
    M, K = x.shape
    n_out = len(outs)
    width = W.shape[0] // n_out
    assert W.shape == (n_out * width, K) and all(t.numel() == M * width for t in outs)
    po = (ctypes.c_void_p * n_out)(*[t.data_ptr() for t in outs])
    for t in outs:
        assert t.is_cuda and t.is_contiguous()
    _check(load_library().dsla_project(int(M), int(K), n_out, int(width), _ptr(x), _ptr(W), _ptr(bias), po, _stream()))


def dsla_attention_prefill(q, k, v, o, scale: float):
    """Causal softmax attention over a prompt (include/dsla.h: dsla_attention_prefill).  q, k, v, o: [B,T,H,d] bf16."""
    B, T, H, d = q.shape
    _check(load_library().dsla_attention_prefill(int(B), int(H), int(d), int(T), _dtype_code(q), float(scale), _ptr(q),
                                                 _ptr(k), _ptr(v), _ptr(o), _stream()))


PLAN_REASONS = ("no pressure", "memory relief", "quality limit", "all converted")


def dsla_rank_layers(sensitivity) -> list:
    """Layer indices in ascending order of sensitivity (include/dsla.h: dsla_rank_layers)."""
    n = len(sensitivity)
    s = (ctypes.c_float * n)(*[float(x) for x in sensitivity])
    order = (ctypes.c_int32 * n)()
    _check(load_library().dsla_rank_layers(n, s, order))
    return list(order)


def dsla_max_conversion_rate(prompt_len: int) -> float:
    return float(load_library().dsla_max_conversion_rate(int(prompt_len)))


def dsla_kv_cache_bytes(n_layers, batch, context, heads, d_head, bytes_per_element) -> int:
    return int(load_library().dsla_kv_cache_bytes(int(n_layers), int(batch), int(context), int(heads), int(d_head),
                                                  int(bytes_per_element)))


def dsla_conversion_plan(order, memory_used, memory_threshold, kv_bytes_per_layer, state_bytes_per_layer, max_rate):
    """Returns (converted layer indices in conversion order, memory use afterwards, reason text)
    (include/dsla.h: dsla_conversion_plan)."""
    n = len(order)
    o = (ctypes.c_int32 * n)(*[int(x) for x in order])
    conv = (ctypes.c_uint8 * n)()
    cnt, after, why = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int32()
    _check(load_library().dsla_conversion_plan(n, o, int(memory_used), int(memory_threshold), int(kv_bytes_per_layer),
                                               int(state_bytes_per_layer), float(max_rate), conv, ctypes.byref(cnt),
                                               ctypes.byref(after), ctypes.byref(why)))
    layers = [l for l in order if conv[l]]
    assert len(layers) == cnt.value
    return layers, int(after.value), PLAN_REASONS[why.value]


def profile_enable(enable: bool, max_records: int = 4096):
    _check(load_library().dsla_profile_enable(1 if enable else 0, int(max_records)))


def profile_collect() -> dict:
    """Returns {kernel name: (total milliseconds, launches)} since the last collect."""
    n = len(KERNEL_NAMES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(load_library().dsla_profile_collect(ms, cnt))
    return {KERNEL_NAMES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}
