"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-side argument checks return the documented codes without a GPU."""
import ctypes
import os
import re

import pytest

import paper_2506_09316_amd as dsla
from paper_2506_09316_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dsla.library_path()):
        from paper_2506_09316_amd import build
        build.build()
    return dsla.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dsla.h")).read()
    return sorted(set(re.findall(r"DSLA_API[^;(]*?\b(dsla_\w+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    for s in range(6):
        assert lib.dsla_status_string(s)


def test_argument_checks_need_no_gpu(lib):
    d = dsla.make_desc(1, 2, 64, 64, io_dtype=0, gate_dtype=0)
    fake = ctypes.c_void_p(4096)
    # NULL state pointer
    assert lib.dsla_state_init(ctypes.byref(d), None, fake, None) == 1
    # unsupported head size
    bad = dsla.make_desc(1, 2, 48, 48, io_dtype=0, gate_dtype=0)
    assert lib.dsla_state_init(ctypes.byref(bad), fake, fake, None) == 3
    # non-positive batch
    bad = dsla.make_desc(0, 2, 64, 64, io_dtype=0, gate_dtype=0)
    assert lib.dsla_decode(ctypes.byref(bad), *([fake] * 9)) == 2
    # misaligned pointer
    odd = ctypes.c_void_p(4100)
    assert lib.dsla_decode(ctypes.byref(d), odd, *([fake] * 8)) == 2
    # chunk lengths other than 32, 64 and 128 are not built
    big = dsla.make_desc(1, 2, 128, 128, io_dtype=0, gate_dtype=0, chunk=48)
    assert lib.dsla_prefill(ctypes.byref(big), 128, *([fake] * 8), None, 0, None) == 3
    # missing workspace when the plan needs one
    seg = dsla.make_desc(1, 2, 64, 64, io_dtype=0, gate_dtype=0, chunk=64, segments=4)
    need = lib.dsla_prefill_workspace_bytes(ctypes.byref(seg), 1024)
    assert need > 0
    assert lib.dsla_prefill(ctypes.byref(seg), 1024, *([fake] * 8), None, 0, None) == 4
    assert lib.dsla_prefill(ctypes.byref(seg), 1024, *([fake] * 8), fake, need - 1, None) == 4
    # gate mode: unknown mode; pre-activation mode needs a finite positive temperature
    bad = dsla.make_desc(1, 2, 64, 64, io_dtype=0, gate_dtype=0, gate_mode=2)
    assert lib.dsla_decode(ctypes.byref(bad), *([fake] * 9)) == 3
    for tau in (0.0, -1.0, float("inf"), float("nan")):
        bad = dsla.make_desc(1, 2, 64, 64, io_dtype=0, gate_dtype=0, gate_mode=1, tau=tau)
        assert lib.dsla_decode(ctypes.byref(bad), *([fake] * 9)) == 2
        assert lib.dsla_prefill_workspace_bytes(ctypes.byref(bad), 1024) == 0
    ignored = dsla.make_desc(1, 2, 64, 64, io_dtype=0, gate_dtype=0, gate_mode=0, tau=0.0)   # tau unused for log gates
    assert lib.dsla_prefill(ctypes.byref(ignored), 0, None, None, None, None, None, fake, fake, None, None, 0, None) == 0
    # packed sequences: the bound of the lengths cannot exceed the total; the offsets are required
    assert lib.dsla_prefill_varlen(ctypes.byref(d), 100, 101, fake, None, None, *([fake] * 8), None, 0, None) == 2
    assert lib.dsla_prefill_varlen(ctypes.byref(d), 100, 50, None, None, None, *([fake] * 8), None, 0, None) == 1
    assert lib.dsla_prefill_varlen(ctypes.byref(d), 2 ** 31, 50, fake, None, None, *([fake] * 8), None, 0, None) == 2
    assert lib.dsla_prefill_varlen(ctypes.byref(d), 0, 0, fake, None, None, None, None, None, None, None, fake, fake,
                                   None, None, 0, None) == 0
    assert lib.dsla_prefill_varlen(ctypes.byref(seg), 4096, 1024, fake, None, None, *([fake] * 8), None, 0, None) == 4
    assert lib.dsla_prefill_varlen(ctypes.byref(d), 100, 50, fake, ctypes.c_void_p(4098), None, *([fake] * 8), None, 0,
                                   None) == 2
    assert lib.dsla_decode_slots(ctypes.byref(d), *([fake] * 5), None, None, *([fake] * 3), None) == 1
    assert lib.dsla_decode_slots(ctypes.byref(d), *([fake] * 5), None, ctypes.c_void_p(4098), *([fake] * 3), None) == 2
    assert lib.dsla_decode_slots(ctypes.byref(d), *([fake] * 5), ctypes.c_void_p(4098), fake, *([fake] * 3), None) == 2
    # T = 0 does nothing and needs no tensors
    assert lib.dsla_prefill(ctypes.byref(d), 0, None, None, None, None, None, fake, fake, None, None, 0, None) == 0
    assert lib.dsla_prefill(ctypes.byref(d), -1, *([fake] * 8), None, 0, None) == 2


def test_projection_argument_checks(lib):
    fake = ctypes.c_void_p(4096)
    outs = (ctypes.c_void_p * 2)(4096, 8192)
    call = lambda M, K, n_out, width, x=fake, W=fake, o=outs: lib.dsla_project(
        ctypes.c_int64(M), K, n_out, width, x, W, None, o, None)
    assert call(0, 128, 2, 128) == 2                       # no rows
    assert call(16, 48, 2, 128) == 3                       # K is not a multiple of 32
    assert call(16, (1 << 21) + 128, 2, 128) == 3          # K beyond the 32-bit offsets of a tile
    assert call(16, 128, 2, 192) == 3                      # width is not a multiple of 128
    assert call(16, 128, 9, 128) == 3                      # more outputs than DSLA_MAX_PROJECTIONS
    assert call(16, 128, 2, 128, x=None) == 1
    assert call(16, 128, 2, 128, W=ctypes.c_void_p(4100)) == 2
    assert call(16, 128, 2, 128, o=(ctypes.c_void_p * 2)(4096, None)) == 1


def test_attention_entropy_argument_checks_and_plan(lib):
    fake = ctypes.c_void_p(4096)
    call = lambda B, H, d, T, io, q=fake, k=fake, o=fake, ws=None, n=0: lib.dsla_attention_entropy(
        B, H, d, T, io, 1.0, q, k, o, ws, n, None)
    assert call(0, 4, 128, 100, 1) == 2
    assert call(2, 4, 128, 0, 1) == 2
    assert call(2, 4, 96, 100, 1) == 3
    assert call(2, 4, 128, 100, 7) == 3
    assert call(2, 4, 128, 100, 1, q=None) == 1
    assert call(2, 4, 128, 100, 1, k=ctypes.c_void_p(4100)) == 2
    # 8 x 32 (batch, head) pairs: two workgroups each -> parts of 4096 keys, 3 floats per part
    assert lib.dsla_attention_entropy_workspace_bytes(8, 32, 128, 8192) == 256 * 2 * 3 * 4
    # 1024 pairs fill the device on their own: no split, no workspace
    assert lib.dsla_attention_entropy_workspace_bytes(32, 32, 128, 8192) == 0
    # a short sequence is not split below 256 keys per workgroup
    assert lib.dsla_attention_entropy_workspace_bytes(1, 2, 64, 600) == 2 * 3 * 3 * 4
    assert call(1, 2, 64, 600, 1) == 4          # workspace needed and missing
    assert lib.dsla_attention_entropy_workspace_bytes(1, 2, 48, 600) == 0


def test_attention_decode_argument_checks_and_plan(lib):
    fake = ctypes.c_void_p(4096)
    call = lambda B, H, d, T, io, q=fake, k=fake, v=fake, o=fake, ws=None, n=0, lens=None: lib.dsla_attention_decode(
        B, H, d, T, io, 1.0, q, k, v, lens, o, ws, n, None)
    assert call(2, 4, 128, 100, 1, lens=ctypes.c_void_p(4098)) == 2
    assert call(2, 0, 128, 100, 1) == 2
    assert call(2, 4, 100, 100, 1) == 3
    assert call(2, 4, 128, 100, 1, v=None) == 1
    assert call(2, 4, 128, 100, 1, o=ctypes.c_void_p(4104)) == 2
    # same split as the entropy kernel, a record of 2 + d floats per part
    assert lib.dsla_attention_decode_workspace_bytes(8, 32, 128, 8192) == 256 * 2 * 130 * 4
    assert lib.dsla_attention_decode_workspace_bytes(32, 32, 128, 8192) == 0
    assert call(8, 32, 128, 8192, 1) == 4


def test_attention_prefill_argument_checks(lib):
    fake = ctypes.c_void_p(4096)
    call = lambda B, H, d, T, io, q=fake, k=fake, v=fake, o=fake: lib.dsla_attention_prefill(
        B, H, d, ctypes.c_int64(T), io, 1.0, q, k, v, o, None)
    assert call(0, 4, 128, 100, 1) == 2
    assert call(2, 4, 100, 100, 1) == 3                  # head size
    assert call(2, 4, 128, 100, 0) == 3                  # fp32 is not built
    assert call(2, 4, 128, 100, 1, k=None) == 1
    assert call(2, 4, 128, 100, 1, o=ctypes.c_void_p(4104)) == 2
    assert call(1, 32, 128, 1 << 19, 1) == 2             # one sequence's tensor reaches 4 GiB: 32-bit byte offsets


def test_varlen_workspace_plan(lib):
    up = lambda n: (n + 255) // 256 * 256
    # 8 sequences, 32 heads; total 32768 tokens, longest 16384.  The segment length follows the total (about one
    # workgroup per compute unit overall): 32768 * 32 / 256 = 4096 tokens, so the longest sequence has 4 segments.
    # Worst case 32768 / 4096 + 8 = 16 segments in all, 8 of them with a successor.
    d = dsla.make_desc(8, 32, 128, 128, io_dtype=1, gate_dtype=1, chunk=64)
    slots = 16 * 32
    want = slots * 2 * 128 * 128 * 4 + up(slots * 2 * 128 * 4) + up(9 * 4) + 256 + up(16 * 8) + up(8 * 8)
    assert lib.dsla_prefill_varlen_workspace_bytes(ctypes.byref(d), 32768, 16384) == want
    # short sequences only: one segment each, no workspace
    assert lib.dsla_prefill_varlen_workspace_bytes(ctypes.byref(d), 2048, 256) == 0
    # equal lengths and a given segment count: the workspace differs from the dense call's only by the lists
    d3 = dsla.make_desc(3, 2, 128, 128, io_dtype=1, gate_dtype=1, chunk=64, segments=3)
    dense = lib.dsla_prefill_workspace_bytes(ctypes.byref(d3), 384)
    packed = lib.dsla_prefill_varlen_workspace_bytes(ctypes.byref(d3), 3 * 384, 384)
    assert dense == 3 * 6 * 2 * 128 * 128 * 4 + up(2 * 6 * 2 * 128 * 4)
    assert packed == 12 * 2 * 2 * 128 * 128 * 4 + up(12 * 2 * 2 * 128 * 4) + up(4 * 4) + 256 + up(12 * 8) + up(9 * 8)


def test_workspace_plan(lib):
    # one segment: no workspace
    d = dsla.make_desc(8, 32, 128, 128, io_dtype=1, gate_dtype=1, chunk=64)
    assert lib.dsla_prefill_workspace_bytes(ctypes.byref(d), 8192) == 0
    # B*H = 32 at T = 16384: 8 segments of both fp32 states plus the decay vectors
    d = dsla.make_desc(1, 32, 128, 128, io_dtype=1, gate_dtype=1, chunk=64)
    n = lib.dsla_prefill_workspace_bytes(ctypes.byref(d), 16384)
    assert n == 8 * 32 * 2 * 128 * 128 * 4 + 7 * 32 * 2 * 128 * 4
    # B*H = 128: two segments, and the pre-pass on the two halves of the first one (3 slots, 2 decay vectors);
    # a caller who asks for two segments gets two slots
    d = dsla.make_desc(4, 32, 128, 128, io_dtype=1, gate_dtype=1, chunk=64)
    assert lib.dsla_prefill_workspace_bytes(ctypes.byref(d), 16384) == 3 * 128 * 2 * 128 * 128 * 4 + 2 * 128 * 2 * 128 * 4
    d = dsla.make_desc(4, 32, 128, 128, io_dtype=1, gate_dtype=1, chunk=64, segments=2)
    assert lib.dsla_prefill_workspace_bytes(ctypes.byref(d), 16384) == 2 * 128 * 2 * 128 * 128 * 4 + 1 * 128 * 2 * 128 * 4


def test_conversion_logic_against_its_oracle(lib):
    """The host-side conversion logic of the library (C++) against the plain Python statement of the same rules:
    the paper's table, rankings of seeded scores with ties, and conversion plans over a sweep of memory situations."""
    import numpy as np
    from oracle import controller as ctl
    for L in (0, 1, 2047, 2048, 3000, 4095, 4096, 8191, 8192, 100000):
        assert dsla.dsla_max_conversion_rate(L) == ctl.max_conversion_rate(L)
    assert dsla.dsla_kv_cache_bytes(32, 8, 8192, 32, 128, 2) == ctl.kv_cache_bytes(32, 8, 8192, 32, 128, 2)
    rng = np.random.default_rng(11)
    for n in (1, 4, 32):
        sens = np.round(rng.uniform(0, 5, n), 1).astype(np.float32)     # rounded: ties occur
        order = dsla.dsla_rank_layers(sens)
        assert order == ctl.rank_layers(sens)
        kv, st = 64 << 20, 4 << 20
        for used_layers in (0, n // 2, n):
            for thr_layers in (0, n // 4, n // 2, n):
                for rate in (0.0, 0.125, 0.25, 0.5, 1.0):
                    used, thr = 1000 + used_layers * kv, 1000 + thr_layers * kv
                    assert dsla.dsla_conversion_plan(order, used, thr, kv, st, rate) == \
                        ctl.conversion_plan(order, used, thr, kv, st, rate)
    # argument errors
    bad = (ctypes.c_int32 * 3)(0, 0, 1)
    conv = (ctypes.c_uint8 * 3)()
    cnt = ctypes.c_int32()
    assert lib.dsla_conversion_plan(3, bad, 10, 5, 2, 1, 1.0, conv, ctypes.byref(cnt), None, None) == 2
    assert lib.dsla_rank_layers(2, (ctypes.c_float * 2)(1.0, float("nan")), (ctypes.c_int32 * 2)()) == 2
