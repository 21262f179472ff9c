#!/usr/bin/env python3
"""Benchmark of the GTO hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic logits already resident
in HBM: for the current and the frozen-reference draft model, row statistics + top-k of every
used draft row, layer-wise expansion, global top-g, target row statistics, Draft Tree Reward and
greedy verification walk; then debiased group-standardised advantages, the clipped surrogate
and its gradient w.r.t. the current draft logits.

Prints ONE JSON line: trees scored per second (value), plus `roofline` for the dominant kernel
(the draft row kernel; algorithmic bytes / HIP-event time measured on the launch stream inside
the timed region) and `cpu_baseline` (the CPU oracle timed on a bounded sample of the same
workload).
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

HBM_PEAK_GBS = 8000.0      # MI355X published peak HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix peak


def bench_fused(args, torch, S, G):
    """The fifth workload: hidden states x LM head on the matrix cores, logits never stored."""
    from paper_2509_22134_amd.pipeline import GtoFusedPath
    dev = torch.device("cuda:0")
    w = S.FUSED_CONFIGS[args.workload]
    if args.roots:
        w = S.scaled(w, R=args.roots)
    t = S.make_fused(w, dev)
    path = GtoFusedPath(R=w.R, d=w.d, k=w.k, g=w.g, V=w.V, hidden=w.hidden, group_size=w.m, device=dev,
                        eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5,
                        flags=0 if args.no_prune else G.GTO_FLAG_TARGET_PRUNE)

    def step():
        path.step(t["H_cur"], t["H_ref"], t["W_draft"], t["W_target"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    G.gto_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    G.gto_profile_enable(False)
    prof = G.gto_profile_read()
    kernels = {n: {"launches": c, "avg_ms": ms / c} for n, (c, ms) in prof.items()}
    dom = "fused_rows_draft"
    flops = 2.0 * w.R * w.rho * w.V * w.hidden
    dom_ms = kernels[dom]["avg_ms"]
    achieved = flops / (dom_ms * 1e-3) / 1e12
    traffic = None               # HBM-side bytes per launch of the dominant kernel, from the rocprofv3 counter runs
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and not args.roots:
        traffic = json.load(open(tpath)).get(f"{dom}:{w.name}")
    out = {
        "metric": "draft trees scored/sec (build+reward+PPO), fused LM head, V=%d" % w.V,
        "value": 2 * w.R / (dt / args.steps), "unit": "trees/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 x bf16 -> f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: R={w.R} hidden={w.hidden} V={w.V} k={w.k} d={w.d} g={w.g} m={w.m}, "
                               "bf16 hidden states x bf16 LM heads, full path, current + reference tree per root",
                   "target_rows": "all used slots" if args.no_prune else "only slots with a kept child",
                   "target_rows_multiplied": [int(path.buf[x]["tree"]["slot_need"].sum().item()) for x in ("cur", "ref")],
                   "draft_rows": w.R * w.rho},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
                     "flops_per_launch": flops, "avg_launch_ms": dom_ms},
        "kernels": kernels,
    }
    if args.cpu_roots > 0:
        import numpy as np
        from oracle import gto_oracle as O
        n = min(2, w.R)
        t0 = time.perf_counter()
        H = {k: t[k][:n].float().cpu().numpy() for k in ("H_cur", "H_ref")}
        Wd, Wt = t["W_draft"].float().cpu().numpy(), t["W_target"].float().cpu().numpy()
        L = {"D_cur": O.fused_logits(H["H_cur"], Wd), "T_cur": O.fused_logits(H["H_cur"], Wt),
             "D_ref": O.fused_logits(H["H_ref"], Wd), "T_ref": O.fused_logits(H["H_ref"], Wt)}
        O.full_path(L["D_cur"], L["T_cur"], L["D_ref"], L["T_ref"], k=w.k, d=w.d, g=w.g, m=1, eta=w.eta, eps=w.eps,
                    delta=w.delta, grad_scale=0.5)
        dtc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2 * n / dtc, "unit": "trees/s", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"first {n} roots (2 trees each, fp64 matmuls through the BLAS numpy links, "
                                         f"then the full path incl. gradient), {dtc:.1f} s"}
    print(json.dumps(out))


def cpu_baseline(w, tens, n_roots, torch):
    """The oracle as it stands, on the first `n_roots` roots of the same tensors."""
    import numpy as np
    from oracle import gto_oracle as O
    host = {n: t[:n_roots].float().cpu().numpy() for n, t in tens.items()}
    m = w.m if n_roots % w.m == 0 else 1
    t0 = time.perf_counter()
    if w.full_path:
        O.full_path(host["D_cur"], host["T_cur"], host["D_ref"], host["T_ref"], k=w.k, d=w.d, g=w.g, m=m,
                    eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5)
        trees, what = 2 * n_roots, "2 trees each, full path incl. gradient"
    else:
        ds = O.draft_row_stats(host["D_cur"], w.k)
        tree = O.select_topg(O.expand_tree(ds["top_tok"], ds["top_logp32"], w.d, w.k), w.g)
        ts = O.target_row_stats(host["T_cur"])
        O.tree_reward(tree, host["T_cur"], ts["t_lse"], w.eta)
        O.accepted_path(tree, ts["t_argmax"], w.d)
        trees, what = n_roots, "1 tree each, build + reward + greedy walk"
    dt = time.perf_counter() - t0
    return {"value": trees / dt, "unit": "trees/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n_roots} roots of the workload ({what}), {dt:.1f} s of single-threaded numpy"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama31_8b")
    ap.add_argument("--roots", type=int, default=0, help="override the number of roots (debug)")
    ap.add_argument("--waves", type=int, default=0, help="wavefronts per row in the row kernels (tuning)")
    ap.add_argument("--no-prune", action="store_true",
                    help="stream every used target row instead of only those the kept tree refers to")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the library's plain copy kernel (4 GiB) so that HBM counters can be scaled")
    ap.add_argument("--group-size", type=int, default=0, help="override m, the roots per advantage group (0 = workload's)")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph and time its replays (kernel durations then come from one "
                         "eager pass after the timed region)")
    ap.add_argument("--chunk-roots", type=int, default=0,
                    help="process the batch in chunks of this many roots (alternating between two streams)")
    ap.add_argument("--one-stream", action="store_true", help="chunked workloads: issue every chunk on one stream")
    ap.add_argument("--cpu-roots", type=int, default=24, help="roots given to the CPU oracle (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import gto_synth as S
    import paper_2509_22134_amd as G
    from paper_2509_22134_amd.pipeline import GtoPath

    if not os.path.exists(G.lib_path()):
        from paper_2509_22134_amd.build import build_lib
        build_lib()
    if args.workload in S.FUSED_CONFIGS:
        bench_fused(args, torch, S, G)
        return
    dev = torch.device("cuda:0")
    w = S.CONFIGS[args.workload]
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    eager_step = step
    if args.graph and n_lanes == 1:
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph):
            eager_step()
        step = hip_graph.replay
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones((1 << 30,), dtype=torch.int32, device=dev)      # 4 GiB read + 4 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            G.gto_calibration_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst
    use_graph = args.graph and n_lanes == 1
    G.gto_profile_enable(n_lanes == 1 and not use_graph)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    G.gto_profile_enable(False)
    if n_lanes > 1 or use_graph:
        # kernels of the two streams overlap in the timed region (and a graph replay carries no events), so the
        # kernels' own durations are taken from one more eager pass that issues every chunk on one stream
        G.gto_profile_enable(True)
        for _ in range(n_chunks):
            path.step(tens["D_cur"], tens["T_cur"], tens.get("D_ref"), tens.get("T_ref"))
        torch.cuda.synchronize()
        G.gto_profile_enable(False)
    prof = G.gto_profile_read()

    trees_per_step = w.R * (2 if w.full_path else 1)
    ms_per_step = dt / args.steps * 1e3
    value = trees_per_step / (dt / args.steps)
    # bytes the forward had to read: every used draft row, and the target rows actually streamed
    row_bytes = w.V * w.elem_bytes
    n_models = 2 if w.full_path else 1
    if args.no_prune:
        target_rows = n_models * R * w.rho
    else:
        target_rows = sum(int(path.buf[t]["tree"]["slot_need"].sum().item()) for t in path.buf)
    fwd_bytes = n_chunks * (n_models * R * w.rho + target_rows) * row_bytes
    kernels = {n: {"launches": c, "avg_ms": ms / c} for n, (c, ms) in prof.items()}
    dom = "row_stats_draft"
    dom_bytes = R * w.rho * w.V * w.elem_bytes          # every used draft row once per launch
    dom_ms = kernels[dom]["avg_ms"]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        traffic = tj.get(f"{dom}:{w.name}")
    out = {
        "metric": "draft trees scored/sec (build+reward+PPO) and achieved HBM GB/s, V=%d" % w.V,
        "value": value, "unit": "trees/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: R={w.R} V={w.V} k={w.k} d={w.d} g={w.g} m={w.m} "
                               f"{w.dtype} logits, " + ("full path, current + reference tree per root"
                                                       if w.full_path else "reward only"),
                   "chunks": n_chunks, "streams": n_lanes,
                   "kernel_durations": "timed region" if (n_lanes == 1 and not use_graph) else "separate one-stream pass after the timed region",
                   "hip_graph": bool(use_graph),
                   "waves_per_row": args.waves or "auto",
                   "target_rows": "all used slots" if args.no_prune else "only slots with a kept child",
                   "target_rows_streamed_per_chunk": target_rows, "draft_rows_per_chunk": n_models * R * w.rho},
        "logit_gb_s": fwd_bytes / (dt / args.steps) / 1e9,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms},
        "kernels": kernels,
    }
    if args.cpu_roots > 0:
        out["cpu_baseline"] = cpu_baseline(w, tens, min(args.cpu_roots, R), torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
