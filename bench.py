#!/usr/bin/env python3
"""Benchmark of the DSLA layer forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints ONE JSON line.  Headline (`value`): prefill throughput in tokens/s of one
Llama-2-7B-shaped DSLA layer (B=1, H=32, d_k=d_v=128, bf16 I/O, fp32 states, chunk 64)
at T=16384; a step is one dsla_prefill over the whole sequence from zero states (the state
initialisation is part of the call: desc.zero_init) with the inputs already resident in HBM; the steps rotate
over three input sets (2.4 GB), so that no step finds parts of its inputs in the 256 MB last-level cache only because
the step before it read the same tensors.  The same line carries the batched-decode measurement
(B=64, 256 single-token steps rotating over 8 independent state sets so that the
256 MB last-level cache cannot hold the states), the roofline objects of the dominant
kernels (durations from HIP events that the library attaches to each kernel launch,
inside the timed region) and the CPU oracle timed on the host cores as a baseline.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
EVENT_SHARE = 8                 # kernel events time every launch of the first 1/EVENT_SHARE of a timed region
EVENT_MIN_STEPS = 8             # ... and of at least this many steps
SETTLE_SECONDS = 0.5            # untimed steps before --warmup


def read_traffic(kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), as recorded in
    profiles/hbm_traffic.txt by hand from the counter runs; None when not recorded."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*%s\s+bytes_per_launch\s*=\s*([0-9.eE+]+)" % re.escape(kernel), line)
        if m:
            return float(m.group(1))
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps first; the clocks and caches of the device need a few dozen to settle")
    ap.add_argument("--T", type=int, default=16384, help="prefill length (default: the headline 16384)")
    ap.add_argument("--segments", type=int, default=0)
    ap.add_argument("--chunk", type=int, default=64)
    ap.add_argument("--decode-steps", type=int, default=1024)
    ap.add_argument("--input-sets", type=int, default=3,
                    help="prefill input sets the steps rotate over, so that no step finds its inputs in the 256 MB "
                         "last-level cache because the step before it read the same tensors (1: one set, as a loop "
                         "over one layer's tensors would)")
    ap.add_argument("--event-steps", type=int, default=0,
                    help="kernel events time the launches of this many steps at the start of each timed region "
                         "(0: an eighth of the region, at least 8 steps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--settle-seconds", type=float, default=SETTLE_SECONDS,
                    help="untimed steps before --warmup (counter runs under rocprofv3 pass 0: every dispatch is slow there)")
    ap.add_argument("--no-calibration-copy", action="store_true",
                    help="skip the plain 256 MiB device copy that gives counter runs a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives); use --gpus 1")

    import numpy as np
    import torch
    import paper_2506_09316_amd as dsla
    import workloads as wl
    from paper_2506_09316_amd.binding import DSLA_BF16

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dsla.load_library()
    dev = "cuda"

    if not args.no_calibration_copy:
        # a plain copy of known size (256 MiB read + 256 MiB written): FETCH_SIZE / WRITE_SIZE of rocprofv3
        # counter runs are scaled by what they report for this kernel
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ prefill
    c = dict(wl.CONFIGS["cfg3_16k"])
    B, H, D, T = c["B"], c["H"], c["dk"], args.T
    x = wl.layer_inputs(c["seed"], B, T, H, D, D, io_dtype="bf16", gate_dtype="bf16", qk_scale=c["qk_scale"])
    xg = {n: torch.from_numpy(a).to(dev).to(torch.bfloat16).contiguous() for n, a in x.items()}
    desc = dsla.make_desc(B, H, D, D, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, gamma=0.5, scale=1.0,
                          chunk=args.chunk, segments=args.segments, zero_init=True)
    # further input sets: the same sequences shifted cyclically along the token axis (same statistics, other memory)
    sets = [xg] + [{n: t.roll(shifts=1 + 4099 * s, dims=1).contiguous() for n, t in xg.items()}
                   for s in range(1, max(1, args.input_sets))]
    S1 = torch.empty(B, H, D, D, device=dev, dtype=torch.float32)
    S2 = torch.empty_like(S1)
    o = torch.empty_like(xg["v"])
    nws = dsla.dsla_prefill_workspace_bytes(desc, T)
    ws = torch.empty(max(nws, 256), dtype=torch.uint8, device=dev)

    def prefill_step(i):
        xs = sets[i % len(sets)]
        dsla.dsla_prefill(desc, T, xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], S1, S2, o, ws if nws else None)

    # Settle phase, fixed and untimed, before the caller's warm-up: the first launches after start-up run slower
    # (clocks ramp up, code objects and page tables are touched for the first time), so a short --warmup alone
    # would time that transient instead of the steady state.
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle_seconds:
        for i in range(20):
            prefill_step(i)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        prefill_step(i)
    torch.cuda.synchronize()
    # Kernel durations come from HIP events inside the timed region, on the launch stream: the library attaches a
    # pair of events to each of its launches (hipExtLaunchKernelGGL: the dispatch itself stamps the start and the
    # end of the kernel, no event packets of their own enter the stream).  A timed step still costs about 8 us
    # (measured: 500 timed steps of 500 against 62: 0.3065 against 0.2993 ms per step), so the launches of the first
    # eighth of the region are timed, all of them.
    ev_steps = args.event_steps if args.event_steps > 0 else max(EVENT_MIN_STEPS, args.steps // EVENT_SHARE)
    ev_steps = max(1, min(args.steps, ev_steps))
    dsla.profile_enable(True, 4 * ev_steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        prefill_step(args.steps - 1 - i)   # the last step runs on set 0, whose results the oracle checks below
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = dsla.profile_collect()
    dsla.profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = B * T / (ms_per_step * 1e-3)

    kern_ms = {k: (v[0] / v[1] if v[1] else None) for k, v in prof.items()}
    loop_ms = kern_ms["prefill_chunk_loop"]
    token_heads = B * T * H
    alg_bytes = 6 * D * 2 * token_heads                    # q k v g1 g2 in, o out, bf16
    C = args.chunk
    alg_flops = (2 * D * (C + 1) + D * (C + 1) + 8 * D * D) * token_heads
    roofline = {
        "kernel": "prefill_chunk_loop", "bound": "hbm",
        "achieved": alg_bytes / (loop_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "traffic": read_traffic("prefill_chunk_loop"),
        "traffic_source": "profiles/hbm_traffic.txt (rocprofv3 --pmc runs of this command, recorded; not measured in this run)",
        "avg_kernel_ms": loop_ms,
        "mfma_tflops_algorithmic": alg_flops / (loop_ms * 1e-3) / 1e12,
        "mfma_frac_of_bf16_peak": alg_flops / (loop_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
    }
    roofline["frac"] = roofline["achieved"] / roofline["peak"]

    out = {
        "metric": "DSLA layer tokens/s (prefill 7B-shape T=16k; decode B=64); % of roofline",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "value = prefill tokens/s of cfg3: B=1 H=32 d_k=d_v=128 T=%d chunk=%d bf16 io, bf16 "
                               "log-gates, fp32 states; step = one prefill call from zero states; the decode part of the "
                               "metric (cfg4, B=64) is under \"decode\"" % (T, C),
                   "segments": args.segments, "input_sets": len(sets), "kernel_events": "all launches of the first %d steps of the timed region, events attached to the dispatches" % ev_steps, "workspace_bytes": nws},
        "roofline": roofline,
        "kernel_ms": {k: v for k, v in kern_ms.items() if v is not None},
        "end_to_end_hbm_frac": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
    }

    # all kernels of a step against the HBM roofline: algorithmic bytes over the sum of their durations
    step_kernel_ms = sum(v for v in kern_ms.values() if v is not None)
    out["step_roofline"] = {"bound": "hbm", "kernels": sorted(k for k, v in kern_ms.items() if v is not None),
                            "achieved": alg_bytes / (step_kernel_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": alg_bytes / (step_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "sum_kernel_ms": step_kernel_ms}
    # results of the last timed step, kept for the comparison with the oracle below
    got = None
    if not args.no_cpu_baseline:
        got = (o.float().cpu().numpy(), S1.cpu().numpy(), S2.cpu().numpy())

    # ------------------------------------------------------------------ batched decode
    del xg, sets, o, ws
    if not args.no_decode:
        c4 = wl.CONFIGS["cfg4"]
        Bd, Hd, Dd, Tp = c4["B"], c4["H"], c4["dk"], c4["T"]
        NSETS = 8
        ddesc = dsla.make_desc(Bd, Hd, Dd, Dd, io_dtype=DSLA_BF16, gate_dtype=DSLA_BF16, gamma=0.5, scale=1.0,
                               chunk=64)
        gen = torch.Generator(device=dev)
        gen.manual_seed(c4["seed"])

        def rnd(shape, scale=1.0, mean=0.0):
            return torch.randn(shape, device=dev, generator=gen, dtype=torch.float32) * scale + mean

        def gates(shape):
            return (-torch.nn.functional.softplus(-rnd(shape, 1.0, 2.0)) / 16.0).to(torch.bfloat16)

        sets = []
        # states pre-populated by a T=2048 prefill per sequence (same value distribution as cfg3)
        pq = rnd((Bd, Tp, Hd, Dd), c4["qk_scale"]).to(torch.bfloat16)
        pk = rnd((Bd, Tp, Hd, Dd), c4["qk_scale"]).to(torch.bfloat16)
        pv = rnd((Bd, Tp, Hd, Dd), c4["qk_scale"]).to(torch.bfloat16)
        pg1, pg2 = gates((Bd, Tp, Hd, Dd)), gates((Bd, Tp, Hd, Dd))
        po = torch.empty_like(pv)
        pws_n = dsla.dsla_prefill_workspace_bytes(ddesc, Tp)
        pws = torch.empty(max(pws_n, 256), dtype=torch.uint8, device=dev)
        for s in range(NSETS):
            a = torch.empty(Bd, Hd, Dd, Dd, device=dev, dtype=torch.float32)
            b = torch.empty_like(a)
            dsla.dsla_state_init(ddesc, a, b)
            # a different roll of the same tokens per set keeps the sets distinct without 8x the inputs
            dsla.dsla_prefill(ddesc, Tp, pq.roll(s, 0), pk.roll(s, 1), pv, pg1, pg2, a, b, po, pws if pws_n else None)
            sets.append((a, b))
        torch.cuda.synchronize()
        t_pre0 = time.perf_counter()
        dsla.dsla_prefill(ddesc, Tp, pq, pk, pv, pg1, pg2, sets[0][0], sets[0][1], po, pws if pws_n else None)
        torch.cuda.synchronize()
        batched_prefill_ms = (time.perf_counter() - t_pre0) * 1e3
        del pq, pk, pv, pg1, pg2, po, pws
        dq = [rnd((Bd, Hd, Dd), c4["qk_scale"]).to(torch.bfloat16) for _ in range(NSETS)]
        dk = [rnd((Bd, Hd, Dd), c4["qk_scale"]).to(torch.bfloat16) for _ in range(NSETS)]
        dv = [rnd((Bd, Hd, Dd), c4["qk_scale"]).to(torch.bfloat16) for _ in range(NSETS)]
        dg1 = [gates((Bd, Hd, Dd)) for _ in range(NSETS)]
        dg2 = [gates((Bd, Hd, Dd)) for _ in range(NSETS)]
        do = torch.empty(Bd, Hd, Dd, device=dev, dtype=torch.bfloat16)

        def decode_steps(n):
            for i in range(n):
                s = i % NSETS
                dsla.dsla_decode(ddesc, dq[s], dk[s], dv[s], dg1[s], dg2[s], sets[s][0], sets[s][1], do)

        decode_steps(64)
        torch.cuda.synchronize()
        nd = args.decode_steps
        dsla.profile_enable(True, max(1, min(nd, args.event_steps if args.event_steps > 0 else nd // EVENT_SHARE)))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        decode_steps(nd)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dprof = dsla.profile_collect()
        dsla.profile_enable(False)
        dec_ms = dprof["decode"][0] / max(dprof["decode"][1], 1)
        dec_bytes = Bd * Hd * (2 * Dd * Dd * 4 * 2 + (4 * Dd + 2 * Dd) * 2)
        out["decode"] = {
            "workload": "cfg4 decode: B=64 H=32 d=128, %d steps rotating over %d state sets" % (nd, NSETS),
            "value": Bd * nd / (t1 - t0), "unit": "tokens/s", "ms_per_step": (t1 - t0) * 1e3 / nd,
            "roofline": {"kernel": "decode", "bound": "hbm", "achieved": dec_bytes / (dec_ms * 1e-3) / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": dec_bytes / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": read_traffic("decode"),
                         "traffic_source": "profiles/hbm_traffic.txt (recorded, not measured in this run)",
                         "avg_kernel_ms": dec_ms},
            "batched_prefill_B64_T2048_ms": batched_prefill_ms,
            "batched_prefill_tokens_per_s": Bd * Tp / (batched_prefill_ms * 1e-3),
        }
        del sets

    # ------------------------------------------------------------------ CPU oracle baseline
    if not args.no_cpu_baseline:
        from oracle import dsla_oracle as orc
        Ts = min(T, 16384)
        xs = {n: a[:, :Ts] for n, a in x.items()}
        t0 = time.perf_counter()
        ro, rS1, rS2 = orc.recurrent(xs["q"], xs["k"], xs["v"], xs["g1"], xs["g2"], 0.5)
        dt = time.perf_counter() - t0
        # the timed steps' own results against the oracle (every head, every token it covered)
        def rel(a, b):
            return float(np.max(np.abs(a - b)) / np.max(np.abs(b)))
        out["check_vs_oracle"] = {"o_max_rel_err": rel(got[0][:, :Ts], ro), "tolerance": 2e-2,
                                  "tokens": Ts, "heads": H}
        if Ts == T:
            out["check_vs_oracle"].update(S1_max_rel_err=rel(got[1], rS1), S2_max_rel_err=rel(got[2], rS2))
        bad = [k for k, v in out["check_vs_oracle"].items() if k.endswith("rel_err") and not v <= 2e-2]
        if bad:
            print(json.dumps(out), flush=True)
            sys.exit("bench.py: results of the timed steps disagree with the oracle: %s" % bad)
        del got, ro
        out["cpu_baseline"] = {"value": B * Ts / dt, "unit": "tokens/s", "cores": orc.threads(), "kind": "oracle",
                               "sample": "prefill workload, first %d tokens of the same inputs, all %d heads, "
                                         "fp64 token-by-token recurrence, %.1f s" % (Ts, H, dt)}
        if not args.no_decode:
            rng = np.random.default_rng(7)
            nds = 16
            dx = {n: rng.standard_normal((64, nds, 32, 128), dtype=np.float32) * 0.088 for n in ("q", "k", "v")}
            dgs = {n: -np.abs(rng.standard_normal((64, nds, 32, 128), dtype=np.float32)) * 0.01 for n in ("g1", "g2")}
            t0 = time.perf_counter()
            orc.recurrent(dx["q"], dx["k"], dx["v"], dgs["g1"], dgs["g2"], 0.5)
            dt = time.perf_counter() - t0
            out["decode"]["cpu_baseline"] = {"value": 64 * nds / dt, "unit": "tokens/s", "cores": orc.threads(),
                                             "kind": "oracle",
                                             "sample": "%d decode steps at B=64 H=32 d=128, %.1f s" % (nds, dt)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
