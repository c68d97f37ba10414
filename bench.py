#!/usr/bin/env python3
"""Benchmark of the HSD batched-verify step on one MI355X.

A step is one whole pass of the hot path (row statistics -> accept / first reject -> residual tile
weights -> inverse-CDF select) through the C ABI over one batch of the headline workload:
B=256 sequences x gamma=8 drafts, V=128256, bf16 logits, T=0.8, with the entropy threshold cycling
through {0.25, 0.5, 0.75} ln V from step to step.  Inputs are synthetic (seeded, LLM-shaped logits)
and resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--steps K] [--warmup W]      the benchmark
  python bench.py --tree 4,4,4,2,2              the same step over token trees (nodes per depth; not the headline)
  python bench.py --copy-calibration            only a plain copy kernel of known size, for scaling the
                                                FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run
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

# HBM traffic of one launch of the dominant kernel on the headline workload, from rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy of known size (see profiles/); None until measured.
# (filter_scan_kernel: measured with --top-k 50 --top-p 0.95.)
MEASURED_TRAFFIC_BYTES = {"row_stats_kernel": 1117785113, "fused_kernel": None, "filter_scan_kernel": 1154513715}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


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
    P = torch.from_numpy(w.target.view(np.int16)).to(dev)
    D = torch.from_numpy(w.draft.view(np.int16)).to(dev)
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

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    hb.hola_profile_enable(True)
    hb.hola_profile_collect()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    stage_ms, stage_n = hb.hola_profile_collect()
    hb.hola_profile_enable(False)
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
    k_ms = stage_ms[0] / max(stage_n[0], 1)
    achieved = k_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    out = {
        "metric": "verified tree nodes/sec + achieved HBM GB/s (% of MI355X peak)",
        "value": round(B * N * args.steps / dt, 1), "unit": "nodes/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"token trees (not the headline workload): B={B}, nodes per depth {widths} (N={N}), V={V} bf16 "
                               f"logits T=0.8, tau cycling (off, 0.25 ln V)",
                   "entry_point": "hola_verify_tree", "parallelism": "single GPU"},
        "stage_ms": {hb.STAGE_NAMES[i]: round(stage_ms[i] / stage_n[i], 5) for i in range(hb.HOLA_N_STAGES) if stage_n[i]},
        "per_threshold": per_tau,
        "roofline": {"bound": "hbm", "kernel": "row_stats_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     # measured for this one shape only (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, see profiles/)
                     "traffic": 1971637248 if (B == 256 and widths == [4, 4, 4, 2, 2]) else None,
                     "algorithmic_bytes_per_launch": int(k_bytes), "avg_launch_ms": round(k_ms, 5)},
    }
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
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-baseline leg")
    ap.add_argument("--copy-calibration", action="store_true")
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
    hb.hola_set_tuning(path={"auto": hb.PATH_AUTO, "split": hb.PATH_SPLIT, "fused": hb.PATH_FUSED}[args.path])
    if args.tree:
        return bench_tree(args)

    t0 = time.perf_counter()
    w = wl.config3(B=args.batch)
    log(f"workload {w.name}: generated in {time.perf_counter() - t0:.1f}s, {w.logit_bytes / 1e9:.3f} GB of logits")
    B, g, V = w.B, w.gamma, w.V
    P = torch.from_numpy(w.target.view(np.int16)).to(dev)
    D = torch.from_numpy(w.draft.view(np.int16)).to(dev)
    tok = torch.from_numpy(w.tokens).to(dev)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    ent = torch.empty((B, g), dtype=torch.float32, device=dev)
    ws = hb.alloc_workspace(hb.hola_workspace_bytes(B, g, V), dev)
    stream = torch.cuda.current_stream()
    taus = w.taus

    def step(i, seed_offset=True):
        hb.hola_verify_ex(target_logits=P, draft_logits=D, draft_tokens=tok, seed=w.seed + (i if seed_offset else 0),
                          B=B, gamma=g, V=V, temperature=w.temperature, entropy_threshold=taus[i % len(taus)],
                          out_accept_len=acc, out_next_token=nxt, out_entropy=ent, workspace=ws, stream=stream,
                          top_k=args.top_k, top_p=args.top_p)

    filtered = (0 < args.top_k < V) or (0.0 < args.top_p < 1.0)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    positions_per_s = B * g * args.steps / dt

    # ---- the same K steps again with HIP events recorded around every kernel on the launch stream
    # (the events cost a few microseconds per kernel, so they stay out of the region `value` comes from)
    hb.hola_profile_enable(True)
    hb.hola_profile_collect()                                # forget anything older
    resid_total = 0
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    stage_ms, stage_n = hb.hola_profile_collect()
    hb.hola_profile_enable(False)

    # bytes the sampler re-reads per step, averaged over the threshold cycle; what the thresholds do to the batch
    per_tau = []
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

    # ---- distribution of single-call times (events on the launch stream around each call)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 200))]
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    call_us = np.sort(np.array([e0.elapsed_time(e1) * 1e3 for e0, e1 in evs]))
    call_dist = {"median": round(float(np.median(call_us)), 1), "p10": round(float(np.percentile(call_us, 10)), 1),
                 "p90": round(float(np.percentile(call_us, 90)), 1), "calls": len(evs)}

    # ---- roofline of the dominant kernel.  Algorithmic bytes: every logit of the gamma draft rows and
    # gamma+1 target rows read once (split path); the fused kernel also reads the stop rows once more.
    pass1_bytes = B * (2 * g + 1) * V * 2
    # Stop rows: a rejection re-reads the target and the draft row; a bonus draw re-reads one slab of the target
    # row (an eighth of it on this shape) when the split-row partials are at hand, the whole row otherwise.
    bonus_row_fraction = 1.0 if (args.path == "fused" or filtered) else 0.125
    stop_bytes = (2 * resid + (B - resid) * bonus_row_fraction) * V * 2
    fused = stage_n[5] > 0
    if fused:
        kname, k_ms, k_bytes = "fused_kernel", stage_ms[5] / stage_n[5], pass1_bytes + stop_bytes
    elif filtered and stage_n[8] > 0:                      # the candidate scan dominates: it reads every row once
        kname, k_ms, k_bytes = "filter_scan_kernel", stage_ms[8] / stage_n[8], pass1_bytes
    elif filtered and stage_n[7] > 0:                      # the per-row keep-set kernel alone (large top_k)
        kname, k_ms, k_bytes = "filter_kernel", stage_ms[7] / stage_n[7], pass1_bytes
    else:
        kname, k_ms, k_bytes = "row_stats_kernel", stage_ms[0] / max(stage_n[0], 1), pass1_bytes
    achieved = k_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(kname),
                "algorithmic_bytes_per_launch": int(k_bytes), "avg_launch_ms": round(k_ms, 5)}
    stages = {hb.STAGE_NAMES[i]: round(stage_ms[i] / stage_n[i], 5) for i in range(hb.HOLA_N_STAGES) if stage_n[i]}
    call_bytes = pass1_bytes + stop_bytes
    call_gbps = call_bytes / (ms_per_step * 1e-3) / 1e9

    out = {
        "metric": "verified draft positions/sec + achieved HBM GB/s (% of MI355X peak)",
        "value": round(positions_per_s, 1), "unit": "positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"cfg3: B={B} gamma={g} V={V} bf16 logits T=0.8, tau cycling (0.25,0.5,0.75) ln V"
                               + (f", top_k={args.top_k} top_p={args.top_p} (not the headline workload)" if filtered else ""),
                   "entry_point": "hola_verify_ex", "kernel_path": "fused" if fused else "split",
                   "parallelism": "single GPU"},
        "hbm_gbps_whole_call": round(call_gbps, 1), "hbm_frac_whole_call": round(call_gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": int(call_bytes),
        "stage_ms": stages,
        "mean_rejections_per_step": round(resid, 1),
        "per_threshold": per_tau,
        "call_us": call_dist,
        "roofline": roofline,
    }

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
        same = same_t = near = 0
        for i, tau in enumerate(taus):
            step(i, seed_offset=False)
            torch.cuda.synchronize()
            same += int((acc.cpu().numpy() == refs[i].accept_len).sum())
            same_t += int((nxt.cpu().numpy() == refs[i].next_token).sum())
            # sequences with a deciding comparison the oracle lists as near-threshold (margin < 1e-6)
            m = np.minimum(np.nan_to_num(refs[i].sample_margin, nan=np.inf),
                           np.minimum(np.nan_to_num(refs[i].gate_margin, nan=np.inf).min(axis=1),
                                      np.nan_to_num(refs[i].ratio_margin, nan=np.inf).min(axis=1)))
            near += int((m < 1e-6).sum())
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
                               "oracle_listed_near_threshold": near}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
