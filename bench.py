#!/usr/bin/env python3
"""Benchmark of the GTO hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic logits already resident
in HBM: for the current and the frozen-reference draft model, row statistics + top-k of every
used draft row, layer-wise expansion, global top-g, target row statistics, Draft Tree Reward and
greedy verification walk; then debiased group-standardised advantages, the clipped surrogate
and its gradient w.r.t. the current draft logits.

Prints ONE JSON line.  Its top-level keys are the headline workload (the third configuration,
LLaMA-3.1-8B-shaped, V = 128256): trees scored per second (value), `roofline` for the dominant
kernel (the draft row kernel; algorithmic bytes / HIP-event time measured on the launch stream
inside the timed region) and `cpu_baseline` (the CPU oracle, fanned out over the machine's host
cores, timed on a bounded sample of the same workload).  `all_configs` carries one entry per
configuration (five, plus the headline workload with one group over the whole batch and the fused
configuration's companion with a correlated target head):
ms/step, trees/s, the dominant kernel's fraction of its roofline, the rows streamed, the
per-kernel durations with their algorithmic bytes or flops, and the oracle's near-tie count on
the sampled roots.

`--workload NAME` measures that one workload only (the form the rocprofv3 commands in profiles/
use); `--headline-only` skips `all_configs`.
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

HBM_PEAK_GBS = 8000.0             # MI355X published peak HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0    # MI355X published dense bf16 matrix peak
TRAFFIC_FILE = os.path.join("profiles", "traffic.json")
HEADLINE = "llama31_8b"


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def traffic_from_profile(kernel, workload):
    """HBM-side bytes per launch from the committed rocprofv3 counter runs (a profiler cannot run inside
    this process); null when the profile does not cover the kernel on this workload."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if not os.path.exists(path):
        return None, None
    tj = json.load(open(path))
    v = tj.get(f"{kernel}:{workload}")
    return v, (f"{TRAFFIC_FILE} ({tj.get('_source', 'rocprofv3 FETCH_SIZE / WRITE_SIZE runs')})" if v is not None else None)


# ----------------------------------------------------------------------------------------------- CPU baseline
def cpu_baseline_streaming(P, w, tens, n_roots):
    """The oracle as it stands over the first `n_roots` roots, one slice of whole groups per worker."""
    n_roots = min(n_roots, tens["D_cur"].shape[0])
    per = max(w.m, (n_roots // max(P.workers(), 1)) // w.m * w.m) if w.full_path else max(1, n_roots // P.workers())
    jobs, off, r0 = [], 0, 0
    while r0 < n_roots:
        r1 = min(r0 + per, n_roots)
        handles = {}
        for name, t in tens.items():
            h = P.arena_put(off, t[r0:r1])
            handles[name] = h
            off += h["nbytes"]
        m = w.m if (r1 - r0) % w.m == 0 else 1
        jobs.append(dict(logits=handles, V=w.V, k=w.k, d=w.d, g=w.g, m=m, eta=w.eta, eps=w.eps, delta=w.delta,
                         full_path=w.full_path))
        r0 = r1
    t0 = time.perf_counter()
    res = P.run(P.timed_full_path, jobs, label=f"cpu_baseline {w.name}", quiet=True)
    dt = time.perf_counter() - t0
    trees = sum(r["trees"] for r in res)
    what = "2 trees each, full path incl. gradient" if w.full_path else "1 tree each, build + reward + greedy walk"
    return {"value": trees / dt, "unit": "trees/s", "cores": P.workers(), "kind": "oracle",
            "sample": f"first {n_roots} roots of the workload ({what}) as {len(jobs)} slices over {P.workers()} "
                      f"worker processes, one per host core of the box's share; {dt:.1f} s wall, "
                      f"{sum(r['seconds'] for r in res):.1f} CPU-s",
            "near_tie_trees": sum(r["near_ties"] for r in res), "trees_sampled": trees}


def cpu_baseline_fused(P, w, t, n_roots, torch):
    off, heads = 0, {}
    for hn in ("W_draft", "W_target"):
        heads[hn] = P.arena_put(off, t[hn].double())
        off += heads[hn]["nbytes"]
    jobs = []
    for r in range(min(n_roots, w.R)):
        hidden = {}
        for hn in ("H_cur", "H_ref"):
            hidden[hn] = P.arena_put(off, t[hn][r:r + 1])
            off += hidden[hn]["nbytes"]
        jobs.append(dict(hidden=hidden, heads=heads, k=w.k, d=w.d, g=w.g, m=1, eta=w.eta, eps=w.eps, delta=w.delta,
                         full_path=True))
    t0 = time.perf_counter()
    res = P.run(P.timed_full_path, jobs, label=f"cpu_baseline {w.name}", quiet=True)
    dt = time.perf_counter() - t0
    trees = sum(r["trees"] for r in res)
    return {"value": trees / dt, "unit": "trees/s", "cores": P.workers(), "kind": "oracle",
            "sample": f"first {len(jobs)} roots (2 trees each: four fp64 matmuls per root through the BLAS numpy "
                      f"links, one thread each, then the full path incl. gradient), one root per worker process "
                      f"over {P.workers()} host cores; {dt:.1f} s wall, {sum(r['seconds'] for r in res):.1f} CPU-s",
            "near_tie_trees": sum(r["near_ties"] for r in res), "trees_sampled": trees}


# ----------------------------------------------------------------------------------------------- streaming workloads
def run_streaming(name, args, steps, warmup, P, torch, S, G, cpu_roots):
    from paper_2509_22134_amd.pipeline import GtoPath
    dev = torch.device("cuda:0")
    w = S.CONFIGS[name]
    if args.roots:
        w = S.scaled(w, R=args.roots)
    if args.group_size:
        w = S.scaled(w, m=args.group_size)
    if args.chunk_roots:
        w = S.scaled(w, chunk_roots=args.chunk_roots)
    R = w.chunk_roots or w.R
    n_chunks = w.R // R
    wr = S.scaled(w, R=R)
    want = ("D_cur", "T_cur", "D_ref", "T_ref") if w.full_path else ("D_cur", "T_cur")
    tens = S.make_logits(wr, dev, want=want)        # one chunk resident; chunks reuse the buffers
    log(f"{name}: inputs generated")
    # a chunked workload alternates its chunks between two streams (each with its own buffers), so that the
    # short per-root kernels of one chunk run under the row streaming of the next
    n_lanes = 2 if (n_chunks > 1 and not args.one_stream) else 1
    paths = [GtoPath(R=R, d=w.d, k=w.k, g=w.g, V=w.V, dtype=w.torch_dtype, group_size=w.m, device=dev,
                     eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, full_path=w.full_path,
                     flags=0 if args.no_prune else G.GTO_FLAG_TARGET_PRUNE, waves_per_row=args.waves)
             for _ in range(n_lanes)]
    path = paths[0]
    streams = [torch.cuda.Stream(device=dev) for _ in range(n_lanes)] if n_lanes > 1 else [None]

    def step():
        if n_lanes == 1:
            for _ in range(n_chunks):
                path.step(tens["D_cur"], tens["T_cur"], tens.get("D_ref"), tens.get("T_ref"))
            return
        start = torch.cuda.current_stream().record_event()
        for c in range(n_chunks):
            st = streams[c % n_lanes]
            if c < n_lanes:
                st.wait_event(start)
            with torch.cuda.stream(st):
                paths[c % n_lanes].step(tens["D_cur"], tens["T_cur"], tens.get("D_ref"), tens.get("T_ref"))
        for st in streams:
            torch.cuda.current_stream().wait_stream(st)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    eager_step = step
    use_graph = args.graph and n_lanes == 1
    if use_graph:
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph):
            eager_step()
        step = hip_graph.replay
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones((1 << 30,), dtype=torch.int32, device=dev)      # 4 GiB read + 4 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            G.gto_calibration_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst
    # In the timed region only the dominant kernel is bracketed by events (two event records per launch leave
    # a few microseconds between consecutive kernels: with all thirteen kernels of a step timed the step is
    # 1.5 % longer); the events come from a pool created here, not in the loop.
    live = n_lanes == 1 and not use_graph
    G.gto_profile_filter("row_stats_draft")
    G.gto_profile_enable(live)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    G.gto_profile_enable(False)
    G.gto_profile_filter(None)
    prof_live = G.gto_profile_read() if live else {}
    # Every kernel's own duration: one more eager pass on one stream after the timed region (kernels of two
    # streams overlap in the timed region, and a graph replay carries no events)
    G.gto_profile_enable(True)
    for _ in range(n_chunks if n_chunks > 1 else 3):
        path.step(tens["D_cur"], tens["T_cur"], tens.get("D_ref"), tens.get("T_ref"))
    torch.cuda.synchronize()
    G.gto_profile_enable(False)
    prof = G.gto_profile_read()
    prof.update(prof_live)          # the dominant kernel: all its launches of the timed region
    kernels = {n: {"launches": c, "avg_ms": ms / c} for n, (c, ms) in prof.items()}

    row_bytes = w.V * w.elem_bytes
    n_models = 2 if w.full_path else 1
    need = [int(path.buf[t]["tree"]["slot_need"].sum().item()) for t in path.buf]
    target_rows = n_models * R * w.rho if args.no_prune else sum(need)
    fwd_bytes = n_chunks * (n_models * R * w.rho + target_rows) * row_bytes
    grad_rows = int((path.grad_slot >= 0).sum().item()) if w.full_path else 0

    def hbm(kname, nbytes):
        if kname in kernels and nbytes > 0:
            k = kernels[kname]
            k["algorithmic_bytes"] = nbytes
            k["gb_s"] = nbytes / (k["avg_ms"] * 1e-3) / 1e9
            k["frac_of_hbm_peak"] = k["gb_s"] / HBM_PEAK_GBS

    hbm("row_stats_draft", R * w.rho * row_bytes)
    hbm("row_stats_target", target_rows / n_models * row_bytes)
    hbm("ppo_bwd", grad_rows * w.V * (w.elem_bytes + 4))
    extras = None
    if w.full_path and not args.no_extras:
        # the token-level loss of Eq. 13 on the same batch (root rows of the current draft and target tensors)
        b = path.buf["cur"]
        loss_rows = torch.empty(R, device=dev); loss = torch.empty(1, device=dev); inv = torch.empty(1, device=dev)
        grad0 = torch.empty((R, w.V), device=dev)
        for it in range(4):
            if it == 1:
                G.gto_profile_enable(True)
            G.gto_token_loss_fwd(path.cfg, tens["D_cur"], tens["T_cur"], b["dstats"], b["tstats"], None, loss_rows, loss, inv)
            G.gto_token_loss_bwd(path.cfg, tens["D_cur"], tens["T_cur"], b["dstats"], b["tstats"], None, inv, 0.5, grad0)
        torch.cuda.synchronize()
        G.gto_profile_enable(False)
        ex = {n: {"launches": c, "avg_ms": ms / c} for n, (c, ms) in G.gto_profile_read().items()}
        for kname, nbytes in (("token_loss_fwd", R * 2 * row_bytes), ("token_loss_bwd", R * (2 * row_bytes + 4 * w.V))):
            ex[kname]["algorithmic_bytes"] = nbytes
            ex[kname]["gb_s"] = nbytes / (ex[kname]["avg_ms"] * 1e-3) / 1e9
            ex[kname]["frac_of_hbm_peak"] = ex[kname]["gb_s"] / HBM_PEAK_GBS
        extras = ex
        del grad0
    dom = "row_stats_draft"
    dom_bytes = kernels[dom]["algorithmic_bytes"]
    dom_ms = kernels[dom]["avg_ms"]
    achieved = kernels[dom]["gb_s"]
    traffic, traffic_source = traffic_from_profile(dom, w.name) if not (args.roots or args.chunk_roots) else (None, None)
    out = {
        "metric": "draft trees scored/sec (build+reward+PPO) and achieved HBM GB/s, V=%d" % w.V,
        "value": w.R * n_models / (dt / steps), "unit": "trees/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: R={w.R} V={w.V} k={w.k} d={w.d} g={w.g} m={w.m} "
                               f"{w.dtype} logits, " + ("full path, current + reference tree per root"
                                                       if w.full_path else "reward only"),
                   "chunks": n_chunks, "streams": n_lanes,
                   "kernel_durations": "row_stats_draft: HIP events over the timed region; the other kernels: "
                                       "three more eager steps after it" if live
                   else "separate one-stream pass after the timed region",
                   "hip_graph": bool(use_graph), "waves_per_row": args.waves or "auto",
                   "target_rows": "all used slots" if args.no_prune else "only slots with a kept child",
                   "target_rows_streamed_per_chunk": target_rows, "draft_rows_per_chunk": n_models * R * w.rho,
                   "gradient_rows_per_chunk": grad_rows},
        "logit_gb_s": fwd_bytes / (dt / steps) / 1e9,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms},
        "kernels": kernels,
    }
    if extras:
        out["token_level_loss"] = extras
    if P is not None and cpu_roots > 0:
        out["cpu_baseline"] = cpu_baseline_streaming(P, wr, tens, cpu_roots)
    del tens, paths, path
    torch.cuda.empty_cache()
    return out


# ----------------------------------------------------------------------------------------------- fused workload
def run_fused(name, args, steps, warmup, P, torch, S, G, cpu_roots, practical_peak=True):
    """The fifth workload: hidden states x LM head on the matrix cores, logits never stored."""
    from paper_2509_22134_amd.pipeline import GtoFusedPath
    dev = torch.device("cuda:0")
    w = S.FUSED_CONFIGS[name]
    if args.roots:
        w = S.scaled(w, R=args.roots)
    t = S.make_fused(w, dev)
    log(f"{name}: inputs generated")
    want_dh = w.w_corr > 0 and not args.no_extras       # the hidden-state backward has rows only with agreeing heads
    path = GtoFusedPath(R=w.R, d=w.d, k=w.k, g=w.g, V=w.V, hidden=w.hidden, group_size=w.m, device=dev,
                        eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5,
                        flags=0 if args.no_prune else G.GTO_FLAG_TARGET_PRUNE, fused_groups=args.fused_groups,
                        fused_layout=args.fused_layout, want_dh=want_dh)
    W_hv = t["W_draft"].t().contiguous() if want_dh else None

    def step():
        path.step(t["H_cur"], t["H_ref"], t["W_draft"], t["W_target"], W_draft_hv=W_hv)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    G.gto_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    G.gto_profile_enable(False)
    prof = G.gto_profile_read()
    kernels = {n: {"launches": c, "avg_ms": ms / c} for n, (c, ms) in prof.items()}
    need = [int(path.buf[x]["tree"]["slot_need"].sum().item()) for x in ("cur", "ref")]
    grad_rows = int((path.grad_slot >= 0).sum().item())
    per_row = 2.0 * w.V * w.hidden

    def mfma(kname, flops):
        if kname in kernels and flops > 0:
            k = kernels[kname]
            k["algorithmic_flops"] = flops
            k["tflop_s"] = flops / (k["avg_ms"] * 1e-3) / 1e12
            k["frac_of_bf16_peak"] = k["tflop_s"] / MFMA_BF16_PEAK_TFLOPS

    mfma("fused_rows_draft", w.R * w.rho * per_row)
    mfma("fused_rows_target", (w.R * w.rho if args.no_prune else sum(need) / 2) * per_row)
    mfma("fused_rows_bwd", grad_rows * per_row)
    mfma("fused_rows_bwd_planes", grad_rows * per_row)
    mfma("fused_dh", grad_rows * per_row)
    dom = "fused_rows_draft"
    flops = kernels[dom]["algorithmic_flops"]
    dom_ms = kernels[dom]["avg_ms"]
    achieved = kernels[dom]["tflop_s"]
    traffic, traffic_source = traffic_from_profile(dom, w.name) if not args.roots else (None, None)
    roof = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
            "traffic_source": traffic_source, "flops_per_launch": flops, "avg_launch_ms": dom_ms}
    if practical_peak:
        # what the in-image bf16 GEMM (torch.matmul) reaches on the same operands and shape, output discarded:
        # the yardstick for what this box's matrix cores sustain on this data
        rows = torch.cat([t["H_cur"][:, 0, 0:1], t["H_cur"][:, 1:].reshape(w.R, -1, w.hidden)], dim=1)
        A = rows.reshape(-1, w.hidden).contiguous()
        Wt = t["W_draft"]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for it in range(4):
            if it == 1:
                ev[0].record()
            out_mm = torch.matmul(A, Wt.t())
            del out_mm
        ev[1].record()
        torch.cuda.synchronize()
        mm_ms = ev[0].elapsed_time(ev[1]) / 3
        roof["practical_peak"] = {"tflop_s": flops / (mm_ms * 1e-3) / 1e12, "avg_ms": mm_ms,
                                  "how": f"torch.matmul of the same [{A.shape[0]}, {w.hidden}] x [{w.hidden}, {w.V}] bf16 "
                                         "operands (library GEMM of the image), mean of 3 launches, bf16 output "
                                         "written and discarded"}
        roof["frac_of_practical_peak"] = achieved / roof["practical_peak"]["tflop_s"]
        del A, rows
    out = {
        "metric": "draft trees scored/sec (build+reward+PPO), fused LM head, V=%d" % w.V,
        "value": 2 * w.R / (dt / steps), "unit": "trees/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: R={w.R} hidden={w.hidden} V={w.V} k={w.k} d={w.d} g={w.g} m={w.m}, "
                               f"bf16 hidden states x bf16 LM heads (fp32 accumulation), target head correlation "
                               f"{w.w_corr}, full path, current + reference tree per root",
                   "target_rows": "all used slots" if args.no_prune else "only slots with a kept child",
                   "target_rows_multiplied": need, "draft_rows": w.R * w.rho, "gradient_rows": grad_rows,
                   "backward": ("empty: the independent second head leaves every accepted path empty, so the timed "
                                "step is forward only" if grad_rows == 0 else
                                f"{grad_rows} (root, step) rows multiplied" + (", logits-row and hidden-state gradients"
                                                                               if want_dh else ""))},
        "roofline": roof,
        "kernels": kernels,
    }
    if P is not None and cpu_roots > 0:
        out["cpu_baseline"] = cpu_baseline_fused(P, w, t, cpu_roots, torch)
    del t, path
    torch.cuda.empty_cache()
    return out


def summary(full):
    """One entry of `all_configs`: the compact form of a workload's line."""
    r = full["roofline"]
    e = {"workload": full["config"]["workload"], "ms_per_step": full["ms_per_step"], "trees_per_s": full["value"],
         "steps": full["steps"], "warmup": full["warmup"],
         "dominant_kernel": r["kernel"], "bound": r["bound"], "achieved": r["achieved"], "unit": r["unit"],
         "frac": r["frac"], "kernels": full["kernels"], "config": {k: v for k, v in full["config"].items() if k != "workload"}}
    if "logit_gb_s" in full:
        e["logit_gb_s"] = full["logit_gb_s"]
    if "practical_peak" in r:
        e["practical_peak"] = r["practical_peak"]
        e["frac_of_practical_peak"] = r["frac_of_practical_peak"]
    if "token_level_loss" in full:
        e["token_level_loss"] = full["token_level_loss"]
    if "cpu_baseline" in full:
        e["cpu_baseline"] = full["cpu_baseline"]
        e["near_tie_trees_in_oracle_sample"] = f"{full['cpu_baseline']['near_tie_trees']} of {full['cpu_baseline']['trees_sampled']}"
    return e


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, help="measure this workload only (default: the headline workload plus "
                                                     "one all_configs entry per configuration)")
    ap.add_argument("--headline-only", action="store_true", help="skip all_configs")
    ap.add_argument("--roots", type=int, default=0, help="override the number of roots (debug)")
    ap.add_argument("--waves", type=int, default=0, help="wavefronts per row in the row kernels (tuning)")
    ap.add_argument("--fused-groups", type=int, default=0, help="fused variant: vocabulary chunks per row block (tuning)")
    ap.add_argument("--fused-layout", type=int, default=0, help="fused variant: workgroups of a group as 0 = 8 row blocks x 4 column tiles, 1 = 4 x 8 (tuning)")
    ap.add_argument("--no-prune", action="store_true",
                    help="stream every used target row instead of only those the kept tree refers to")
    ap.add_argument("--no-extras", action="store_true", help="skip the token-level loss and the hidden-state backward")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the library's plain copy kernel (4 GiB) so that HBM counters can be scaled")
    ap.add_argument("--group-size", type=int, default=0, help="override m, the roots per advantage group (0 = workload's)")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph and time its replays (kernel durations then come from one "
                         "eager pass after the timed region)")
    ap.add_argument("--chunk-roots", type=int, default=0,
                    help="process the batch in chunks of this many roots (alternating between two streams)")
    ap.add_argument("--one-stream", action="store_true", help="chunked workloads: issue every chunk on one stream")
    ap.add_argument("--cpu-roots", type=int, default=128, help="roots given to the CPU oracle (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    # the oracle's worker processes are forked before this process makes its first GPU call
    P = None
    if args.cpu_roots > 0:
        from oracle import pool as P
        P.start()

    import torch

    import gto_synth as S
    import paper_2509_22134_amd as G

    if not os.path.exists(G.lib_path()):
        from paper_2509_22134_amd.build import build_lib
        build_lib()

    def run(name, steps, warmup, cpu_roots):
        if name in S.FUSED_CONFIGS:
            return run_fused(name, args, steps, warmup, P, torch, S, G, min(cpu_roots, 16))
        return run_streaming(name, args, steps, warmup, P, torch, S, G, cpu_roots)

    try:
        if args.workload:
            out = run(args.workload, args.steps, args.warmup, args.cpu_roots)
        else:
            out = run(HEADLINE, args.steps, args.warmup, args.cpu_roots)
            if not args.headline_only:
                entries = []
                plan = (("tiny", 50, 5, 4), ("vicuna13b", 20, 3, 128), (HEADLINE, 0, 0, 0), ("qwen3_8b", 5, 2, 64),
                        ("llama33_70b_fused", 3, 1, 16), ("llama33_70b_fused_corr", 3, 1, 0))
                for name, steps, warmup, cpu_roots in plan:
                    if name == HEADLINE:
                        entries.append(summary(out))
                        continue
                    log(f"all_configs: {name}")
                    entries.append(summary(run(name, steps, warmup, cpu_roots if args.cpu_roots > 0 else 0)))
                # the headline workload once more with the advantage standardised over the whole batch
                # (one group of R roots) instead of groups of m
                if not args.group_size:
                    log(f"all_configs: {HEADLINE}, one group over the batch")
                    args.group_size = S.CONFIGS[HEADLINE].R
                    e = summary(run(HEADLINE, 5, 2, 0))
                    args.group_size = 0
                    e["workload"] += " [advantage standardised over the batch: one group of R roots]"
                    entries.insert(3, e)
                out["all_configs"] = entries
    finally:
        if P is not None:
            P.stop()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
