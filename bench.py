#!/usr/bin/env python3
"""Benchmark of the HSD batched-verify step on one MI355X.

A step is one whole pass of the hot path (row statistics -> accept / first reject -> residual tile
weights -> inverse-CDF select) through the C ABI over one batch of the headline workload:
B=256 sequences x gamma=8 drafts, V=128256, bf16 logits, T=0.8, with the entropy threshold cycling
through {0.25, 0.5, 0.75} ln V from step to step.  Inputs are synthetic (seeded, LLM-shaped logits)
and resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--steps K] [--warmup W]      the benchmark (headline workload, configuration 3)
  python bench.py --config {1,2,4,5}            the other named workloads (labelled, not the headline): 1 and 2 rotate
                                                through more distinct inputs than the 256 MB last-level cache holds and
                                                also give the cache-resident figure; 4 is the two-level hierarchy
                                                (level-0 positions over the whole call); 5 the 9.4 GB float workload
  python bench.py --tree 4,4,4,2,2              the same step over token trees (nodes per depth; not the headline)
  python bench.py --read-ceiling                what a read-only streaming kernel shaped like the statistics pass
                                                reaches on this machine (plain loads, non-temporal loads, and
                                                non-temporal loads carrying the pass's arithmetic)
  python bench.py --copy-calibration            only a plain copy kernel of known size, for scaling the
                                                FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run

Protocol.  Before the warm-up an untimed pre-roll of `settle_calls` steps lets the clocks settle (the first
launches after an idle period run up to 25 % slower); then W warm-up steps, then exactly K timed steps between two
synchronisations give `value`.  The roofline leg is separate: at least 200 steps with HIP events recorded by the
library around every kernel on the launch stream; `roofline.achieved` uses the MEDIAN launch of the dominant kernel.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
SETTLE_CALLS = 200              # untimed steps before the warm-up (disclosed in the output)
ROOFLINE_MIN_LAUNCHES = 200
STAGE_ROW_STATS, STAGE_FUSED, STAGE_TAIL, STAGE_FILTER, STAGE_SCAN, STAGE_PROBE = 0, 5, 6, 7, 8, 10

# HBM traffic of one launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs scaled by a
# plain copy of known size (see profiles/).  Keyed by the library version the counters were read with and by the
# workload: a figure is reported only for the very kernels it was measured on, otherwise null.
MEASURED_TRAFFIC_BYTES = {
    ("hola-verify 0.2 (gfx950)", "cfg3", "row_stats_kernel"): 1117891619,
    ("hola-verify 0.2 (gfx950)", "cfg5", "row_stats_kernel"): 9438836104,
    ("hola-verify 0.2 (gfx950)", "cfg3 top_k=50 top_p=0.95", "filter_scan_kernel"): 1154944365,
    ("hola-verify 0.2 (gfx950)", "tree 4,4,4,2,2", "row_stats_kernel"): 1971627097,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def _dist(us):
    import numpy as np
    us = np.sort(np.asarray(us, dtype=np.float64))
    return {"median": round(float(np.median(us)), 2), "p10": round(float(np.percentile(us, 10)), 2),
            "p90": round(float(np.percentile(us, 90)), 2), "mean": round(float(us.mean()), 2), "n": int(us.size)}


def _event_timed(step, n, stream):
    """Microseconds of n single calls, each bracketed by events on the launch stream, issued back to back."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) * 1e3 for e0, e1 in evs]


def _kernel_launches(hb, step, n):
    """Per-launch milliseconds by stage over n steps, from the library's own events around each kernel."""
    import torch
    hb.hola_profile_enable(True)
    hb.hola_profile_collect()                                # forget anything older
    per_stage = {}
    done = 0
    while done < n:                                          # collect in slices so that the event pool stays small
        m = min(100, n - done)
        for i in range(done, done + m):
            step(i)
        torch.cuda.synchronize()
        for st, ms in hb.hola_profile_collect_launches():
            per_stage.setdefault(st, []).append(ms)
        done += m
    hb.hola_profile_enable(False)
    return per_stage


def _settle(step, n=SETTLE_CALLS):
    import torch
    for i in range(n):
        step(i)
    torch.cuda.synchronize()


def _timed(step, steps, warmup):
    import torch
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def _roofline(hb, per_stage, stage, kname, k_bytes, traffic_key):
    import numpy as np
    ms = np.asarray(per_stage.get(stage, [0.0]), dtype=np.float64)
    med = float(np.median(ms))
    achieved = k_bytes / (med * 1e-3) / 1e9 if med > 0 else 0.0
    return {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES.get((hb.hola_version(), traffic_key, kname)),
            "algorithmic_bytes_per_launch": int(k_bytes), "launch_ms_median": round(med, 5),
            "launch_ms_mean": round(float(ms.mean()), 5), "launch_ms_p10": round(float(np.percentile(ms, 10)), 5),
            "launch_ms_p90": round(float(np.percentile(ms, 90)), 5), "launches": int(ms.size),
            "statistic": "median launch of the kernel, HIP events on the launch stream"}


def _host_info():
    """The host the CPU baseline ran on: logical CPUs visible and the processor's model name."""
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "cpu_model": model}


def _to_dev(a, dev="cuda:0"):
    import numpy as np
    import torch
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)


def _base_line(metric, value, unit, steps, warmup, ms_per_step, workload, extra_cfg=None):
    cfg = {"workload": workload, "parallelism": "single GPU"}
    cfg.update(extra_cfg or {})
    return {"metric": metric, "value": round(value, 1), "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
            "settle_calls": SETTLE_CALLS, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None,
            "dtype": "f32",                                   # arithmetic of the path: fp32 terms, fp64 sums and decisions
            "data": "synthetic", "config": cfg}


# ----------------------------------------------------------------------------------------------------------------
def copy_calibration() -> int:
    """Launch the library's plain copy kernel on 1 GiB a few times (nothing else touches the GPU)."""
    import torch
    from paper_2506_18952_amd import binding as hb
    n = 1 << 30
    src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(5):
        hb.hola_copy_bytes(dst, src, n)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration_bytes_per_launch": n, "launches": 5}), flush=True)
    return 0


def read_ceiling(args) -> int:
    """A read-only kernel with the statistics pass's launch shape over a buffer the size of the headline workload's
    logits (4352 rows of 256 512 bytes, two workgroups per row): the practical ceiling beside the published peak."""
    import numpy as np
    import torch
    from paper_2506_18952_amd import binding as hb
    row_bytes, rows, nsplit = 128256 * 2, 4352, 2
    nbytes = row_bytes * rows
    block_bytes = ((row_bytes // 16 + nsplit - 1) // nsplit + 255) // 256 * 256 * 16
    g = torch.Generator(device="cuda:0")
    g.manual_seed(1)
    # bf16 patterns of moderate logits (exponent arguments stay small for the arithmetic variant)
    src = (torch.randn(nbytes // 2, device="cuda:0", generator=g) * 2.0).to(torch.bfloat16)
    stream = torch.cuda.current_stream()
    out = {}
    variants = (("plain_loads", False, False), ("nontemporal_loads", True, False), ("nontemporal_loads_with_pass_arithmetic", True, True))
    for name, nt, ar in variants:
        def step(i, nt=nt, ar=ar):
            hb.hola_read_probe(src, nbytes, block_bytes, nt, ar, stream=stream)
        _settle(step)
        per = _kernel_launches(hb, step, max(args.steps, ROOFLINE_MIN_LAUNCHES))
        ms = np.asarray(per[STAGE_PROBE])
        med = float(np.median(ms))
        out[name] = {"GB/s": round(nbytes / (med * 1e-3) / 1e9, 1), "frac_of_peak": round(nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "launch_us_median": round(med * 1e3, 2), "launch_us_p10": round(float(np.percentile(ms, 10)) * 1e3, 2),
                     "launch_us_p90": round(float(np.percentile(ms, 90)) * 1e3, 2), "launches": int(ms.size)}
    print(json.dumps({"read_ceiling": out, "bytes_per_launch": nbytes, "workgroups": -(-nbytes // block_bytes),
                      "block_bytes": block_bytes, "peak_GB/s": HBM_PEAK_GBPS, "settle_calls": SETTLE_CALLS,
                      "kernel": "read_probe_kernel (hola_read_probe)"}), flush=True)
    return 0


def bench_tree(args) -> int:
    """The verify step over token trees: B sequences of one tree shape on 128256-wide bf16 rows, thresholds cycling
    through (off, 0.25 ln V).  A step is one hola_verify_tree call; the unit of work is a tree node."""
    import numpy as np
    import torch
    from paper_2506_18952_amd import binding as hb
    from paper_2506_18952_amd import workloads as wl
    dev = "cuda:0"
    widths = [int(x) for x in args.tree.split(",")]
    t0 = time.perf_counter()
    w = wl.tree_case(args.batch, widths, 128256, dtype="bf16", temperature=0.8, zipf_slope=1.2, peak_prob=0.3, case_id=795)
    log(f"workload {w.name}: generated in {time.perf_counter() - t0:.1f}s, {w.logit_bytes / 1e9:.3f} GB of logits")
    B, N, V = w.B, w.N, w.V
    P, D = _to_dev(w.target), _to_dev(w.draft)
    tok, par = torch.from_numpy(w.node_token).to(dev), torch.from_numpy(w.node_parent).to(dev)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, N), dtype=torch.int32, device=dev)
    ent = torch.empty((B, N), dtype=torch.float32, device=dev)
    ws = hb.alloc_workspace(hb.hola_tree_workspace_bytes(B, N, V), dev)
    stream = torch.cuda.current_stream()
    taus = [-1.0, float(np.float32(0.25 * np.log(V)))]

    def step(i, seed_offset=True):
        hb.hola_verify_tree(P, D, tok, par, w.seed + (i if seed_offset else 0), B, N, V, w.temperature, taus[i % len(taus)],
                            acc, nxt, ws, out_path=path, out_entropy=ent, stream=stream)

    _settle(step)
    dt = _timed(step, args.steps, args.warmup)
    ms_per_step = dt * 1e3 / args.steps
    per_stage = _kernel_launches(hb, step, max(args.steps, ROOFLINE_MIN_LAUNCHES))
    per_tau = []
    for i in range(len(taus)):
        step(i)
        torch.cuda.synchronize()
        a_np = acc.cpu().numpy()
        per_tau.append({"tau": round(taus[i], 4), "depth_hist": np.bincount(a_np, minlength=len(widths) + 1).tolist(),
                        "emitted_tokens": int(a_np.sum()) + B})
    # algorithmic bytes of the statistics pass: every target row, and the draft rows of contexts with children
    used = int(sum(1 for c in range(N) if (w.node_parent[0] == c - 1).any()))
    k_bytes = B * (used + N + 1) * V * 2
    out = _base_line("verified tree nodes/sec + achieved HBM GB/s (% of MI355X peak)", B * N * args.steps / dt, "nodes/s",
                     args.steps, args.warmup, ms_per_step,
                     f"token trees (not the headline workload): B={B}, nodes per depth {widths} (N={N}), V={V} bf16 "
                     f"logits T=0.8, tau cycling (off, 0.25 ln V)", {"entry_point": "hola_verify_tree", "logit_dtype": "bf16"})
    out["stage_ms"] = {hb.STAGE_NAMES[s]: round(float(np.median(v)), 5) for s, v in sorted(per_stage.items())}
    out["per_threshold"] = per_tau
    out["call_us"] = _dist(_event_timed(step, 200, stream))
    out["roofline"] = _roofline(hb, per_stage, STAGE_ROW_STATS, "row_stats_kernel", k_bytes,
                                "tree " + args.tree if B == 256 else "")
    if not args.no_cpu:
        from oracle import hola_oracle as orc
        threads = orc.max_threads()
        n = min(B, 64)                                          # a slice of the batch: a few seconds of oracle time
        t0 = time.perf_counter()
        refs = [orc.verify_tree(w.target[:n], w.draft[:n], w.node_token[:n], w.node_parent[:n], w.seed, w.temperature, tau,
                                num_threads=threads) for tau in taus]
        cdt = time.perf_counter() - t0
        same = near = 0
        for i in range(len(taus)):
            step(i, seed_offset=False)
            torch.cuda.synchronize()
            ok = (acc.cpu().numpy()[:n] == refs[i].accept_len) & (nxt.cpu().numpy()[:n] == refs[i].next_token) \
                & (path.cpu().numpy()[:n] == refs[i].path).all(axis=1)
            same += int(ok.sum())
            m = np.nanmin(np.c_[refs[i].gate_margin, refs[i].ratio_margin, refs[i].sample_margin, np.full(n, np.inf)], axis=1)
            near += int((m < 1e-6).sum())
        out["cpu_baseline"] = {"value": round(n * N * len(taus) / cdt, 1), "unit": "nodes/s", "cores": threads, "kind": "oracle",
                               "sample": f"the first {n} sequences of the same workload at each of the {len(taus)} thresholds "
                                         f"({cdt:.2f}s wall); float64 C oracle, OpenMP over sequences",
                               "agree_path_and_next_token": f"{same}/{n * len(taus)}", "oracle_listed_near_threshold": near}
    print(json.dumps(out), flush=True)
    return 0


# ----------------------------------------------------------------------------------------------------------------
def _one_level_runner(hb, w, P, D, tok, rt, stream, tau):
    """step(i) for one hola_verify_ex call per step on device tensors that may hold several input sets: set k is
    rows [k*B, (k+1)*B) of P, D, tok, and step i uses set i mod n_sets."""
    import torch
    B, g, V = w.B, w.gamma, w.V
    n_sets = P.shape[0] // B
    acc = torch.empty(B, dtype=torch.int32, device=P.device)
    nxt = torch.empty(B, dtype=torch.int32, device=P.device)
    ent = torch.empty((B, g), dtype=torch.float32, device=P.device)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes_ex(B, g, V), P.device)
    views = [(P[k * B:(k + 1) * B], D[k * B:(k + 1) * B], tok[k * B:(k + 1) * B], None if rt is None else rt[k * B:(k + 1) * B])
             for k in range(n_sets)]

    def make(rotate):
        def step(i):
            p, d, t, r = views[i % n_sets] if rotate else views[0]
            hb.hola_verify_ex(target_logits=p, draft_logits=d, draft_tokens=t, seed=w.seed + i, B=B, gamma=g, V=V,
                              temperature=w.temperature, entropy_threshold=tau, out_accept_len=acc, out_next_token=nxt,
                              out_entropy=ent, workspace=ws, stream=stream, row_temperature=r)
        return step
    return make, (acc, nxt, ent)


def bench_config(args) -> int:
    """Configurations 1, 2, 4 and 5 (not the headline): whole-call times by events around single calls issued back
    to back, the statistics kernel's median launch, and the algorithmic bytes the call has to read."""
    import numpy as np
    import torch
    from paper_2506_18952_amd import binding as hb
    from paper_2506_18952_amd import workloads as wl
    dev = "cuda:0"
    c = args.config
    stream = torch.cuda.current_stream()
    t0 = time.perf_counter()
    n_calls = max(args.steps, ROOFLINE_MIN_LAUNCHES)
    if c in (1, 2):
        # more distinct input sets than the 256 MB last-level cache holds: 256 x 1.15 MB / 8 x 45 MB
        n_sets = 256 if c == 1 else 8
        base = wl.config1() if c == 1 else wl.config2()
        B = base.B
        w = (wl.config1 if c == 1 else wl.config2)(seqs=range(B * n_sets))
        w.B = B
        log(f"workload {base.name} x {n_sets} input sets: generated in {time.perf_counter() - t0:.1f}s, "
            f"{w.logit_bytes / 1e6:.0f} MB of logits")
        g, V, es = w.gamma, w.V, (2 if w.dtype == "bf16" else 4)
        P, D, tok = _to_dev(w.target), _to_dev(w.draft), _to_dev(w.tokens)
        tau = base.taus[0]
        make, (acc, nxt, ent) = _one_level_runner(hb, w, P, D, tok, None, stream, tau)
        res = {}
        for label, rotate in (("rotating_inputs", True), ("cache_resident", False)):
            step = make(rotate)
            _settle(step)
            dt = _timed(step, args.steps, args.warmup)
            res[label] = {"ms_per_step": dt * 1e3 / args.steps, "call_us": _dist(_event_timed(step, n_calls, stream)),
                          "per_stage": _kernel_launches(hb, step, n_calls)}
        step = make(True)
        resid = 0
        for i in range(n_sets):
            step(i)
            torch.cuda.synchronize()
            resid += int((acc.cpu().numpy() < g).sum())
        resid /= n_sets
        pass1 = B * (2 * g + 1) * V * es
        call_bytes = pass1 + 2 * resid * V * es + (B - resid) * V * es * 0.125   # a bonus draw re-reads one slab (an eighth or less)
        rot = res["rotating_inputs"]
        out = _base_line("verified draft positions/sec + achieved HBM GB/s (% of MI355X peak)", B * g / (rot["ms_per_step"] * 1e-3),
                         "positions/s", args.steps, args.warmup, rot["ms_per_step"],
                         f"cfg{c} (not the headline workload): B={B} gamma={g} V={V} {w.dtype} logits T={w.temperature}, "
                         f"tau=0.5 ln V; {n_sets} distinct input sets ({w.logit_bytes / 1e6:.0f} MB) used in rotation",
                         {"entry_point": "hola_verify_ex", "logit_dtype": w.dtype, "headline": False})
        for label in res:
            r = res[label]
            med = r["call_us"]["median"]
            out[label] = {"call_us": r["call_us"], "ms_per_step_back_to_back": round(r["ms_per_step"], 5),
                          "positions_per_s_at_median_call": round(B * g / (med * 1e-6), 1),
                          "algorithmic_GB/s_at_median_call": round(call_bytes / (med * 1e-6) / 1e9, 1),
                          "frac_of_peak": round(call_bytes / (med * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                          "stage_ms_median": {hb.STAGE_NAMES[s]: round(float(np.median(v)), 5) for s, v in sorted(r["per_stage"].items())}}
        out["algorithmic_bytes_per_step"] = int(call_bytes)
        out["ideal_us_at_peak"] = round(call_bytes / HBM_PEAK_GBPS / 1e3, 3)
        out["roofline"] = _roofline(hb, rot["per_stage"], STAGE_ROW_STATS, "row_stats_kernel", pass1, "")
        oracle_case = (base, [tau])
    elif c == 5:
        w = wl.config5(B=args.batch5)
        log(f"workload {w.name}: generated in {time.perf_counter() - t0:.1f}s, {w.logit_bytes / 1e9:.3f} GB of logits")
        B, g, V, es = w.B, w.gamma, w.V, 4
        P, D, tok, rt = _to_dev(w.target), _to_dev(w.draft), _to_dev(w.tokens), _to_dev(w.row_temperature)
        tau = w.taus[0]
        make, (acc, nxt, ent) = _one_level_runner(hb, w, P, D, tok, rt, stream, tau)
        step = make(False)
        _settle(step, 40)
        steps = min(args.steps, 60)
        dt = _timed(step, steps, min(args.warmup, 10))
        ms_per_step = dt * 1e3 / steps
        calls = _dist(_event_timed(step, 60, stream))
        per_stage = _kernel_launches(hb, step, 60)
        step(0)
        torch.cuda.synchronize()
        a_np = acc.cpu().numpy()
        stoch = w.row_temperature > 0
        resid = int(((a_np < g) & stoch).sum())
        bonus = int(((a_np >= g) & stoch).sum())
        pass1 = B * (2 * g + 1) * V * es
        call_bytes = pass1 + (2 * resid + bonus * 0.0625) * V * es          # greedy rows re-read nothing; a slab is 1/16 here
        out = _base_line("verified draft positions/sec + achieved HBM GB/s (% of MI355X peak)", B * g * steps / dt, "positions/s",
                         steps, min(args.warmup, 10), ms_per_step,
                         f"cfg5 (not the headline workload): B={B} gamma={g} V={V} f32 logits, rows below {B // 2} greedy, "
                         f"the rest T=0.7, tau=0.5 ln V, one call with per-row temperatures",
                         {"entry_point": "hola_verify_ex", "logit_dtype": "f32", "headline": False})
        out["settle_calls"] = 40
        out["call_us"] = calls
        out["hbm_gbps_whole_call"] = round(call_bytes / (ms_per_step * 1e-3) / 1e9, 1)
        out["hbm_frac_whole_call"] = round(call_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        out["algorithmic_bytes_per_step"] = int(call_bytes)
        out["stage_ms"] = {hb.STAGE_NAMES[s]: round(float(np.median(v)), 5) for s, v in sorted(per_stage.items())}
        out["rejections"] = resid
        out["roofline"] = _roofline(hb, per_stage, STAGE_ROW_STATS, "row_stats_kernel", pass1, "cfg5" if args.batch5 == 1024 else "")
        oracle_case = None
        if not args.no_cpu:
            from oracle import hola_oracle as orc
            threads = orc.max_threads()
            lo, hi = B // 2 - 32, B // 2 + 32                                # 64 sequences across the greedy boundary
            t0 = time.perf_counter()
            orc.verify(w.target[lo:hi], w.draft[lo:hi], w.tokens[lo:hi], w.seed, w.temperature, tau,
                       row_temperature=w.row_temperature[lo:hi], seq_base=lo, num_threads=threads)
            cdt = time.perf_counter() - t0
            out["cpu_baseline"] = {"value": round(64 * g / cdt, 1), "unit": "positions/s", "cores": threads, "kind": "oracle",
                                   "sample": f"sequences {lo}..{hi - 1} of the same workload ({cdt:.2f}s wall); float64 C oracle"}
    else:                                                                    # c == 4: the two-level hierarchy
        w = wl.config4()
        log(f"workload {w.name}: generated in {time.perf_counter() - t0:.1f}s")
        ms = [_to_dev(m) for m in w.models]
        B, g, V, es = w.B, w.gamma, w.V, 2
        n = len(ms)
        out_tok = torch.empty((B, g + n - 1), dtype=torch.int32, device=dev)
        acc = torch.empty(B, dtype=torch.int32, device=dev)
        nxt = torch.empty(B, dtype=torch.int32, device=dev)
        ent = torch.empty((n - 1, B, g + n - 2), dtype=torch.float32, device=dev)
        ws = hb.alloc_workspace(hb.hola_hsd_workspace_bytes(n, B, g, V), dev)
        tok = _to_dev(w.tokens)

        def step(i):
            hb.hola_hsd_verify(ms, tok, w.seed + i, B, g, V, w.temperature, w.taus, out_tok, acc, nxt, ent, ws, stream=stream)

        _settle(step)
        dt = _timed(step, args.steps, args.warmup)
        ms_per_step = dt * 1e3 / args.steps
        calls = _dist(_event_timed(step, n_calls, stream))
        per_stage = _kernel_launches(hb, step, n_calls)
        step(0)
        torch.cuda.synchronize()
        len2 = (out_tok.cpu().numpy() >= 0).sum(axis=1)                      # drafts handed to the second level
        a2 = acc.cpu().numpy()
        rows1 = B * (2 * g + 1)
        rows2 = int((len2 + 1).sum())                                        # target rows j <= len; the draft statistics are reused
        resid2 = int((a2 < len2).sum())
        call_bytes = (rows1 + rows2) * V * es + B * 1.5 * V * es + (2 * resid2 + (B - resid2) * 0.125) * V * es
        out = _base_line("verified draft positions/sec + achieved HBM GB/s (% of MI355X peak)", B * g * args.steps / dt,
                         "positions/s", args.steps, args.warmup, ms_per_step,
                         f"cfg4 (not the headline workload): two-level hierarchy, B={B} gamma={g} V={V} bf16 logits T=1, "
                         f"tau=(0.4, 0.6) ln V; value = level-0 drafted positions over the whole two-level call",
                         {"entry_point": "hola_hsd_verify", "logit_dtype": "bf16", "headline": False})
        out["call_us"] = calls
        out["algorithmic_bytes_per_step"] = int(call_bytes)
        out["algorithmic_bytes_note"] = ("rows streamed by both levels (the middle model's statistics are reused) plus the stop "
                                         "rows; the first level's stop rows counted at 1.5 rows per sequence")
        out["hbm_gbps_whole_call"] = round(call_bytes / (ms_per_step * 1e-3) / 1e9, 1)
        out["hbm_frac_whole_call"] = round(call_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        out["stage_ms_median_per_launch"] = {hb.STAGE_NAMES[s]: round(float(np.median(v)), 5) for s, v in sorted(per_stage.items())}
        out["second_level_target_rows"] = rows2
        l1 = np.asarray(per_stage[STAGE_ROW_STATS][0::2])                     # launches alternate: level 1, level 2
        out["roofline"] = _roofline(hb, {STAGE_ROW_STATS: list(l1)}, STAGE_ROW_STATS, "row_stats_kernel", rows1 * V * es, "")
        out["roofline"]["note"] = "the first level's statistics launch"
        oracle_case = None
        if not args.no_cpu:
            from oracle import hola_oracle as orc
            threads = orc.max_threads()
            t0 = time.perf_counter()
            ref = orc.hsd_verify(w.models, w.tokens, w.seed, w.temperature, w.taus, num_threads=threads)
            cdt = time.perf_counter() - t0
            hb.hola_hsd_verify(ms, tok, w.seed, B, g, V, w.temperature, w.taus, out_tok, acc, nxt, ent, ws, stream=stream)
            torch.cuda.synchronize()
            out["cpu_baseline"] = {"value": round(B * g / cdt, 1), "unit": "positions/s", "cores": threads, "kind": "oracle",
                                   "sample": f"all {B} sequences, both levels ({cdt:.2f}s wall); float64 C oracle",
                                   "agree_accept_len": f"{int((acc.cpu().numpy() == ref.accept_len).sum())}/{B}",
                                   "agree_next_token": f"{int((nxt.cpu().numpy() == ref.next_token).sum())}/{B}"}
    if oracle_case is not None and not args.no_cpu:
        from oracle import hola_oracle as orc
        base, taus = oracle_case
        threads = orc.max_threads()
        reps = 20 if c == 1 else 3
        t0 = time.perf_counter()
        for _ in range(reps):
            orc.verify(base.target, base.draft, base.tokens, base.seed, base.temperature, taus[0], num_threads=threads)
        cdt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": round(base.B * base.gamma / cdt, 1), "unit": "positions/s", "cores": threads, "kind": "oracle",
                               "sample": f"the first input set, mean of {reps} oracle calls ({cdt * 1e3:.1f} ms each); float64 C oracle"}
    print(json.dumps(out), flush=True)
    return 0


# ----------------------------------------------------------------------------------------------------------------
def bench_variant(args) -> int:
    """The headline shape on inputs or through an entry point other than the headline's (labelled so)."""
    import numpy as np
    import torch
    from paper_2506_18952_amd import binding as hb
    from paper_2506_18952_amd import workloads as wl
    dev = "cuda:0"
    w = wl.config3(B=args.batch)
    B, g, V = w.B, w.gamma, w.V
    tgt, drf, toks = w.target, w.draft, w.tokens
    what = "hola_verify_literal_ex (every non-gated position takes a draw from its target row)"
    if args.variant in ("padded", "masked"):
        tgt, drf, toks = tgt.copy(), drf.copy(), toks.copy()
        mask = np.zeros(V, bool)
        mask[V - 256:] = True
        if args.variant == "masked":
            mask |= np.random.default_rng(1).random(V) < 0.3
        tgt[..., mask] = np.uint16(0xff80)                       # bf16 -inf
        drf[..., mask] = np.uint16(0xff80)
        ok = np.flatnonzero(~mask)
        toks = ok[np.random.default_rng(2).integers(0, ok.size, size=toks.shape)].astype(np.int32)
        what = ("the last 256 vocabulary entries of every row at -inf" if args.variant == "padded"
                else "30 % of the vocabulary entries (and the last 256) at -inf")
    two = args.variant == "two-streams"
    if two:
        what = ("two independent batches of the headline shape in flight: calls issued alternately on two streams, each batch "
                "with inputs, outputs and workspace of its own (1.1 GB of logits each); value = both batches' positions")
    sets = []
    for k in range(2 if two else 1):
        sets.append(dict(P=_to_dev(tgt), D=_to_dev(drf), tok=_to_dev(toks),
                         acc=torch.empty(B, dtype=torch.int32, device=dev), nxt=torch.empty(B, dtype=torch.int32, device=dev),
                         ent=torch.empty((B, g), dtype=torch.float32, device=dev),
                         ws=hb.alloc_workspace(hb.hola_workspace_bytes_ex(B, g, V), dev),
                         stream=torch.cuda.Stream() if two else torch.cuda.current_stream()))
    out = torch.empty((B, g), dtype=torch.int32, device=dev)
    stream = sets[0]["stream"]
    taus = w.taus
    ns = len(sets)

    def step(i):
        q = sets[i % ns]
        common = dict(target_logits=q["P"], draft_logits=q["D"], draft_tokens=q["tok"], seed=w.seed + i, B=B, gamma=g, V=V,
                      temperature=w.temperature, entropy_threshold=taus[(i // ns) % len(taus)], out_entropy=q["ent"],
                      workspace=q["ws"], stream=q["stream"])
        if args.variant == "literal":
            hb.hola_verify_literal_ex(out_tokens=out, out_verifier_calls=q["acc"], **common)
        else:
            hb.hola_verify_ex(out_accept_len=q["acc"], out_next_token=q["nxt"], **common)

    _settle(step)
    dt = _timed(step, args.steps, args.warmup)
    per_stage = _kernel_launches(hb, step, max(args.steps, ROOFLINE_MIN_LAUNCHES))
    line = _base_line("verified draft positions/sec + achieved HBM GB/s (% of MI355X peak)", B * g * args.steps / dt, "positions/s",
                      args.steps, args.warmup, dt * 1e3 / args.steps,
                      f"cfg3 shape (not the headline workload): B={B} gamma={g} V={V} bf16 logits T={w.temperature}, tau cycling "
                      f"(0.25,0.5,0.75) ln V; {what}",
                      {"entry_point": "hola_verify_literal_ex" if args.variant == "literal" else "hola_verify_ex", "logit_dtype": "bf16"})
    line["stage_ms"] = {hb.STAGE_NAMES[s_]: round(float(np.median(v)), 5) for s_, v in sorted(per_stage.items())}
    line["stage_ms_statistic"] = "median launch"
    rows = B * ((2 * g) if args.variant == "literal" else (2 * g + 1))
    line["roofline"] = _roofline(hb, per_stage, STAGE_ROW_STATS, "row_stats_kernel", rows * V * 2, "")
    if two:
        line["hbm_frac_whole_call"] = round(rows * V * 2 * args.steps / dt / 1e9 / HBM_PEAK_GBPS, 4)
        line["hbm_frac_whole_call_note"] = "the statistics pass's bytes alone over the step time (stop rows not counted)"
        line["roofline"]["note"] = "the two batches' launches run side by side, each on part of the chip: the kernel's own rate is the headline line's"
        line["call_us"] = None
    else:
        line["call_us"] = _dist(_event_timed(step, max(args.steps, ROOFLINE_MIN_LAUNCHES), stream))
    print(json.dumps(line), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--batch", type=int, default=256, help="sequences (256 = the headline workload)")
    ap.add_argument("--path", choices=["auto", "split", "fused"], default="auto", help="kernel path (auto: library's choice)")
    ap.add_argument("--top-k", type=int, default=0, help="top-k filter on both models (0: off; not the headline workload)")
    ap.add_argument("--top-p", type=float, default=0.0, help="top-p filter on both models (0: off; not the headline workload)")
    ap.add_argument("--tree", type=str, default="", help="token trees with this many nodes per depth, e.g. 4,4,4,2,2 "
                                                          "(hola_verify_tree; not the headline workload)")
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5], help="named workload (3 = the headline)")
    ap.add_argument("--batch5", type=int, default=1024, help=argparse.SUPPRESS)
    ap.add_argument("--variant", choices=["literal", "padded", "masked", "two-streams"], default="",
                    help="not the headline workload: the headline shape through hola_verify_literal_ex (Equation (1) taken "
                         "literally), or through hola_verify_ex with the last 256 vocabulary entries of every row at -inf "
                         "(padded) / 30 %% of the entries at -inf (masked), or two independent batches of the headline shape in flight on two "
                         "streams (two-streams)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-baseline leg")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--read-ceiling", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build is one-GPU only (sharding by sequence is a design note, not code); "
            "run with --gpus 1")
        return 2

    import numpy as np
    import torch
    from paper_2506_18952_amd import binding as hb
    from paper_2506_18952_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    hb.lib()                                                 # fails loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        return copy_calibration()
    if args.read_ceiling:
        return read_ceiling(args)
    hb.hola_set_tuning(path={"auto": hb.PATH_AUTO, "split": hb.PATH_SPLIT, "fused": hb.PATH_FUSED}[args.path])
    if args.tree:
        return bench_tree(args)
    if args.variant:
        return bench_variant(args)
    if args.config != 3:
        return bench_config(args)

    t0 = time.perf_counter()
    w = wl.config3(B=args.batch)
    log(f"workload {w.name}: generated in {time.perf_counter() - t0:.1f}s, {w.logit_bytes / 1e9:.3f} GB of logits")
    B, g, V = w.B, w.gamma, w.V
    P, D, tok = _to_dev(w.target), _to_dev(w.draft), _to_dev(w.tokens)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    ent = torch.empty((B, g), dtype=torch.float32, device=dev)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes_ex(B, g, V, args.top_k, args.top_p), dev)
    stream = torch.cuda.current_stream()
    taus = w.taus

    def step(i, seed_offset=True):
        hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed + (i if seed_offset else 0),
                          B=B, gamma=g, V=V, temperature=w.temperature, entropy_threshold=taus[i % len(taus)],
                          out_accept_len=acc, out_next_token=nxt, out_entropy=ent, workspace=ws, stream=stream,
                          top_k=args.top_k, top_p=args.top_p)

    filtered = (0 < args.top_k < V) or (0.0 < args.top_p < 1.0)

    # ---- untimed pre-roll (clocks), W warm-up steps, then the timed region: exactly K steps
    _settle(step)
    dt = _timed(step, args.steps, args.warmup)
    ms_per_step = dt * 1e3 / args.steps
    positions_per_s = B * g * args.steps / dt

    # ---- at least 200 steps with HIP events recorded around every kernel on the launch stream
    # (the events cost a few microseconds per kernel, so they stay out of the region `value` comes from)
    per_stage = _kernel_launches(hb, step, max(args.steps, ROOFLINE_MIN_LAUNCHES))

    # bytes the sampler re-reads per step, averaged over the threshold cycle; what the thresholds do to the batch
    per_tau = []
    resid_total = 0
    for i in range(len(taus)):
        step(i)
        torch.cuda.synchronize()
        a_np, h_np = acc.cpu().numpy(), ent.cpu().numpy()
        resid_total += int((a_np < g).sum())
        per_tau.append({"tau": round(float(taus[i]), 4),
                        "accept_len_hist": np.bincount(a_np, minlength=g + 1).tolist(),
                        "gate_fire_rate": round(float((h_np < np.float32(taus[i])).mean()), 4),
                        "mean_entropy": round(float(h_np.mean()), 4)})
    resid = resid_total / len(taus)

    # ---- distribution of single-call times (events on the launch stream around each call, issued back to back)
    call_dist = _dist(_event_timed(step, max(args.steps, ROOFLINE_MIN_LAUNCHES), stream))

    # ---- roofline of the dominant kernel.  Algorithmic bytes: every logit of the gamma draft rows and
    # gamma+1 target rows read once (split path); the fused kernel also reads the stop rows once more.
    pass1_bytes = B * (2 * g + 1) * V * 2
    # Stop rows: a rejection re-reads the target and the draft row; a bonus draw re-reads one slab of the target
    # row (an eighth of it on this shape) when the split-row partials are at hand, the whole row otherwise.
    bonus_row_fraction = 1.0 if (args.path == "fused" or filtered) else 0.125
    stop_bytes = (2 * resid + (B - resid) * bonus_row_fraction) * V * 2
    fused = STAGE_FUSED in per_stage
    wkey = "cfg3" + (f" top_k={args.top_k} top_p={args.top_p}" if filtered else "") if B == 256 else ""
    if fused:
        roofline = _roofline(hb, per_stage, STAGE_FUSED, "fused_kernel", pass1_bytes + stop_bytes, wkey)
    elif filtered and STAGE_SCAN in per_stage:              # the candidate scan dominates: it reads every row once
        roofline = _roofline(hb, per_stage, STAGE_SCAN, "filter_scan_kernel", pass1_bytes, wkey)
    elif filtered and STAGE_FILTER in per_stage:            # the per-row keep-set kernel alone (large top_k)
        roofline = _roofline(hb, per_stage, STAGE_FILTER, "filter_kernel", pass1_bytes, wkey)
    else:
        roofline = _roofline(hb, per_stage, STAGE_ROW_STATS, "row_stats_kernel", pass1_bytes, wkey)
    call_bytes = pass1_bytes + stop_bytes
    call_gbps = call_bytes / (ms_per_step * 1e-3) / 1e9

    out = _base_line("verified draft positions/sec + achieved HBM GB/s (% of MI355X peak)", positions_per_s, "positions/s",
                     args.steps, args.warmup, ms_per_step,
                     f"cfg3: B={B} gamma={g} V={V} bf16 logits T=0.8, tau cycling (0.25,0.5,0.75) ln V"
                     + (f", top_k={args.top_k} top_p={args.top_p} (not the headline workload)" if filtered else ""),
                     {"entry_point": "hola_verify_ex", "kernel_path": "fused" if fused else "split", "logit_dtype": "bf16"})
    out.update({
        "hbm_gbps_whole_call": round(call_gbps, 1), "hbm_frac_whole_call": round(call_gbps / HBM_PEAK_GBPS, 4),
        "hbm_frac_whole_call_at_median_call": round(call_bytes / (call_dist["median"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": int(call_bytes),
        "stage_ms": {hb.STAGE_NAMES[s]: round(float(np.median(v)), 5) for s, v in sorted(per_stage.items())},
        "stage_ms_statistic": "median launch",
        "mean_rejections_per_step": round(resid, 1),
        "per_threshold": per_tau,
        "call_us": call_dist,
        "roofline": roofline,
    })

    if not args.no_cpu:
        # The float64 oracle as it stands, on the same workload: all B sequences at each of the thresholds.
        from oracle import hola_oracle as orc
        threads = orc.max_threads()
        t0 = time.perf_counter()
        if filtered:
            refs = [orc.verify_filtered(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, top_k=args.top_k,
                                        top_p=args.top_p if 0.0 < args.top_p < 1.0 else 1.0, num_threads=threads)
                    for tau in taus]
        else:
            refs = [orc.verify(w.target, w.draft, w.tokens, w.seed, w.temperature, tau, num_threads=threads) for tau in taus]
        cdt = time.perf_counter() - t0
        same = same_t = near = unlisted_diff = 0
        for i, tau in enumerate(taus):
            step(i, seed_offset=False)
            torch.cuda.synchronize()
            ok_a = acc.cpu().numpy() == refs[i].accept_len
            ok_t = nxt.cpu().numpy() == refs[i].next_token
            same += int(ok_a.sum())
            same_t += int(ok_t.sum())
            # sequences with a deciding comparison the oracle lists as near-threshold (margin < 1e-6)
            m = np.minimum(np.nan_to_num(refs[i].sample_margin, nan=np.inf),
                           np.minimum(np.nan_to_num(refs[i].gate_margin, nan=np.inf).min(axis=1),
                                      np.nan_to_num(refs[i].ratio_margin, nan=np.inf).min(axis=1)))
            near += int((m < 1e-6).sum())
            unlisted_diff += int((~(ok_a & ok_t) & ~(m < 1e-6)).sum())   # differences the parity bar does not allow: must be 0
        n = B * len(taus)
        # the same oracle on one thread, on a slice of the batch (a second or two)
        n1 = min(B, 32)
        t0 = time.perf_counter()
        if filtered:
            orc.verify_filtered(w.target[:n1], w.draft[:n1], w.tokens[:n1], w.seed, w.temperature, taus[0], top_k=args.top_k,
                                top_p=args.top_p if 0.0 < args.top_p < 1.0 else 1.0, num_threads=1)
        else:
            orc.verify(w.target[:n1], w.draft[:n1], w.tokens[:n1], w.seed, w.temperature, taus[0], num_threads=1)
        cdt1 = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(n * g / cdt, 1), "unit": "positions/s", "cores": threads,
                               "single_thread_value": round(n1 * g / cdt1, 1),
                               "kind": "oracle",
                               "sample": f"all {B} sequences of the same workload at each of the {len(taus)} thresholds "
                                         f"({len(taus)} oracle calls, {cdt:.2f}s wall, {cdt * threads:.0f} core-seconds); "
                                         f"float64 C oracle, OpenMP over sequences",
                               "agree_accept_len": f"{same}/{n}", "agree_next_token": f"{same_t}/{n}",
                               "oracle_listed_near_threshold": near, "differences_outside_the_listed": unlisted_diff,
                               "host": _host_info()}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
