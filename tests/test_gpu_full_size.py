"""Parity at the full sizes of the five configurations, in the launch configuration bench.py times
(target-row pruning on; the fourth configuration in 256-root chunks alternating between two streams).

The oracle runs over the batch on CPU-only worker processes (oracle/pool.py), one slice of whole advantage
groups per job, so that every stage - row statistics, tree, reward, verification walk, advantage, surrogate
and gradient rows - is compared through the oracle's own functions, for every root of configurations 2 and
3 and for whole groups of every chunk of configuration 4 and of the fused configuration.  Each test prints
and asserts how many trees the end-to-end stage (stage 3, pure fp64 oracle) actually compared."""
import time

import numpy as np
import pytest
import torch

import gpu_util as U
import gto_synth as S
import oracle_jobs as J
import paper_2509_22134_amd as G
from paper_2509_22134_amd.pipeline import GtoFusedPath, GtoPath

pytestmark = pytest.mark.gpu
GRAD_SCALE = 0.5


def _say(msg):
    print(msg, flush=True)


def _properties(w, path, tag="cur"):
    """Invariants that hold at any size, checked on every root."""
    b = path.buf[tag]
    R = path.cfg.R
    m = torch.from_numpy(U.used_mask(R, w.d, w.k)).to(b["dstats"]["row_lse"].device)
    ds, tr, rw = b["dstats"], b["tree"], b["reward"]
    assert bool((ds["row_lse"][m] >= ds["row_max"][m]).all())
    tt = ds["top_tok"][m]
    assert bool(((tt >= 0) & (tt < w.V)).all())
    lp = ds["top_logp"][m]
    assert bool((lp <= 0).all()) and bool((lp[:, :-1] >= lp[:, 1:]).all())
    assert bool((tr["n_sel"] == min(w.g, w.C)).all())
    assert bool((tr["sel_score"][:, :-1] >= tr["sel_score"][:, 1:]).all())
    idx = torch.arange(w.g, device=tr["sel_parent"].device)[None, :]
    assert bool((tr["sel_parent"] < idx).all())
    aux = rw["reward_aux"]
    n_leaves = rw["n_leaves"].float()
    assert bool((aux[:, 1] <= aux[:, 0] + 1e-5).all())
    assert bool((aux[:, 0] <= aux[:, 1] + torch.log(n_leaves) / w.eta + 1e-5).all())
    assert bool((aux[:, 3] <= w.d + 1e-4).all()) and bool((aux[:, 2] <= aux[:, 1] + 1e-6).all())
    assert bool((aux[:, 3] <= tr["n_sel"].float() + 1e-4).all())       # reward <= number of selected nodes
    assert bool(((rw["path_len"] >= 0) & (rw["path_len"] <= w.d)).all())


def _collect(results, what):
    bad = [r for r in results if not r["ok"]]
    for r in bad[:3]:
        _say(f"  FAILED slice of roots {r['roots']}:\n{r['err']}")
    assert not bad, f"{what}: {len(bad)} of {len(results)} slices disagree with the oracle"
    tot = {k: sum(r.get(k, 0) for r in results) for k in ("n_trees", "n_ambig", "n_clear", "n_same", "grad_rows",
                                                           "path_rows", "dh_rows")}
    tot["ppo_e2e"] = sum(1 for r in results if r.get("ppo_e2e"))
    tot["slices"] = len(results)
    tot["cpu_s"] = sum(r["seconds"] for r in results)
    return tot


def _streaming_jobs(P, w, tens, path, slices, V, K_batch_roots, base_root=0):
    """Copy the logits of the root slices into the arena and build one job per slice.  `slices` are ranges
    of roots of `tens`, each a whole number of groups."""
    jobs, off = [], 0
    for sl in slices:
        roots = list(sl)
        handles = {}
        for name, t in tens.items():
            h = P.arena_put(off, t[sl.start:sl.stop])
            handles[name] = h
            off += h["nbytes"]
        jobs.append(dict(w=w, V=V, logits=handles, rows=None, ppo=w.full_path,
                         bundle=U.bundle_np(path, roots, with_ppo=w.full_path),
                         grad_scale=U.slice_grad_scale(GRAD_SCALE, len(roots), K_batch_roots)))
    return jobs


@pytest.mark.parametrize("name", ["vicuna13b", "llama31_8b"])
def test_full_size_every_root_through_the_oracle(gpu_device, oracle_workers, name):
    P = oracle_workers
    w = S.CONFIGS[name]
    _say(f"full size {name}: R={w.R} V={w.V} k={w.k} d={w.d} g={w.g} m={w.m}, every root, {P.workers()} oracle workers")
    want = ("D_cur", "T_cur", "D_ref", "T_ref") if w.full_path else ("D_cur", "T_cur")
    tens = S.make_logits(w, gpu_device, want=want)
    path = GtoPath(R=w.R, d=w.d, k=w.k, g=w.g, V=w.V, dtype=w.torch_dtype, group_size=w.m, device=gpu_device,
                   eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=GRAD_SCALE, full_path=w.full_path,
                   flags=G.GTO_FLAG_TARGET_PRUNE)
    path.step(tens["D_cur"], tens["T_cur"], tens.get("D_ref"), tens.get("T_ref"))
    torch.cuda.synchronize()
    _say("  GPU path done")
    _properties(w, path, "cur")
    if w.full_path:
        _properties(w, path, "ref")
    # host memory stays bounded: the batch goes through the arena in passes of 16 slices of one group each
    per_job, per_pass = w.m, w.m * P.workers()
    results, t0 = [], time.time()
    for p0 in range(0, w.R, per_pass):
        slices = [range(s, min(s + per_job, w.R)) for s in range(p0, min(p0 + per_pass, w.R), per_job)]
        jobs = _streaming_jobs(P, w, tens, path, slices, w.V, w.R)
        results += P.run(J.streaming_slice, jobs, label=f"{name} roots {p0}..{min(p0 + per_pass, w.R) - 1}")
    tot = _collect(results, name)
    _say(f"  {name}: {tot['n_trees']} trees through the oracle in {time.time() - t0:.0f} s "
         f"({tot['cpu_s']:.0f} CPU-s): stage 3 (pure fp64 oracle): {tot['n_clear']} trees clear of rounding, all "
         f"identical; {tot['n_ambig']} with a near tie, of which {tot['n_same'] - tot['n_clear']} identical too" + (f"; surrogate end to end in {tot['ppo_e2e']}/{tot['slices']} groups; "
                              f"{tot['grad_rows']} gradient rows of {tot['path_rows']} path rows" if w.full_path else ""))
    assert tot["n_trees"] == w.R * (2 if w.full_path else 1)
    assert tot["n_clear"] >= 0.9 * tot["n_trees"], "stage 3 must cover nearly every tree"
    if w.full_path:
        # batch loss = mean over the K groups of the oracle's group losses on the GPU's inputs
        lg = np.concatenate([r["loss_group"] for r in results])
        assert len(lg) == w.R // w.m
        np.testing.assert_allclose(path.ppo["loss"].cpu().numpy()[0], float(lg.mean()), rtol=1e-5, atol=1e-7)
        assert tot["grad_rows"] > 0 and tot["ppo_e2e"] >= 0.5 * tot["slices"]
    del tens, path
    torch.cuda.empty_cache()


def test_full_size_chunked_two_stream_schedule(gpu_device, oracle_workers):
    """Fourth configuration: 2048 roots as 8 chunks of 256, alternating between two streams exactly as
    bench.py issues them.  Every chunk has its own data and output buffers here, so that all eight results
    survive the step; each chunk is compared (a) bit for bit with the same chunk issued alone on one stream
    and (b) with the oracle on two whole groups."""
    P = oracle_workers
    w = S.CONFIGS["qwen3_8b"]
    R, n_chunks = w.chunk_roots, w.R // w.chunk_roots
    _say(f"full size {w.name}: {n_chunks} chunks of {R} roots on two streams, V={w.V} k={w.k} d={w.d} g={w.g}")
    mk = lambda: GtoPath(R=R, d=w.d, k=w.k, g=w.g, V=w.V, dtype=w.torch_dtype, group_size=w.m, device=gpu_device,
                         eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=GRAD_SCALE, flags=G.GTO_FLAG_TARGET_PRUNE)
    chunks, paths = [], []
    for c in range(n_chunks):
        wc = S.scaled(w, R=R, seed=w.seed + 1000 * c, chunk_roots=0)
        chunks.append(S.make_logits(wc, gpu_device))
        paths.append(mk())
        _say(f"  chunk {c}: inputs generated")
    streams = [torch.cuda.Stream(device=gpu_device) for _ in range(2)]
    torch.cuda.synchronize()
    start = torch.cuda.current_stream().record_event()
    for c in range(n_chunks):
        st = streams[c % 2]
        if c < 2:
            st.wait_event(start)
        with torch.cuda.stream(st):
            t = chunks[c]
            paths[c].step(t["D_cur"], t["T_cur"], t["D_ref"], t["T_ref"])
    for st in streams:
        torch.cuda.current_stream().wait_stream(st)
    torch.cuda.synchronize()
    _say("  two-stream step done")
    alone = mk()
    wr = S.scaled(w, R=R)
    rng = np.random.default_rng(4)
    jobs = []
    off = 0
    for c in range(n_chunks):
        t = chunks[c]
        alone.step(t["D_cur"], t["T_cur"], t["D_ref"], t["T_ref"])
        torch.cuda.synchronize()
        for tag in ("cur", "ref"):
            for grp in ("dstats", "pool", "tree", "reward"):
                for n, x in alone.buf[tag][grp].items():
                    assert torch.equal(x, paths[c].buf[tag][grp][n]), (c, tag, grp, n)
            need = alone.buf[tag]["tree"]["slot_need"].bool()
            for n, x in alone.buf[tag]["tstats"].items():
                assert torch.equal(x[need], paths[c].buf[tag]["tstats"][n][need]), (c, tag, n)
        for n, x in alone.ppo.items():
            assert torch.equal(x, paths[c].ppo[n]), (c, n)
        assert torch.equal(alone.adv, paths[c].adv) and torch.equal(alone.grad_slot, paths[c].grad_slot)
        live = alone.grad_slot >= 0
        assert torch.equal(alone.grad_rows[live], paths[c].grad_rows[live]), c
        _properties(wr, paths[c], "cur")
        _properties(wr, paths[c], "ref")
        groups = sorted(rng.choice(R // w.m, size=2, replace=False).tolist())
        for gi in groups:
            sl = range(gi * w.m, (gi + 1) * w.m)
            handles = {}
            for name, x in t.items():
                h = P.arena_put(off, x[sl.start:sl.stop])
                handles[name] = h
                off += h["nbytes"]
            jobs.append(dict(w=wr, V=w.V, logits=handles, rows=None, ppo=True,
                             bundle=U.bundle_np(paths[c], list(sl)),
                             grad_scale=U.slice_grad_scale(GRAD_SCALE, w.m, R)))
        _say(f"  chunk {c}: two-stream result identical to the one-stream result; groups {groups} go to the oracle")
    results = P.run(J.streaming_slice, jobs, label=w.name)
    tot = _collect(results, w.name)
    _say(f"  {w.name}: {tot['n_trees']} trees through the oracle ({tot['cpu_s']:.0f} CPU-s): stage 3: {tot['n_clear']} "
         f"clear of rounding, all identical; {tot['n_ambig']} with a near tie, of which {tot['n_same'] - tot['n_clear']} "
         f"identical too; surrogate end to end in {tot['ppo_e2e']}/{tot['slices']} groups; {tot['grad_rows']} gradient rows")
    assert tot["n_trees"] == 2 * 2 * w.m * n_chunks and tot["n_clear"] >= 0.9 * tot["n_trees"]
    assert tot["grad_rows"] > 0
    del chunks, paths, alone
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,n_groups", [("llama33_70b_fused", 4), ("llama33_70b_fused_corr", 4)])
def test_full_size_fused_whole_groups_through_the_oracle(gpu_device, oracle_workers, name, n_groups):
    """Fifth configuration at its real shape (and its companion with a correlated target head, whose accepted
    paths are not empty, so that the backward multiplies real rows): whole groups of 8 roots through the
    oracle (one fp64 matmul per root and tensor), including gradient rows and hidden-state gradient rows."""
    P = oracle_workers
    w = S.FUSED_CONFIGS[name]
    _say(f"full size {name}: R={w.R} V={w.V} k={w.k} d={w.d} g={w.g} hidden={w.hidden} corr={w.w_corr}")
    t = S.make_fused(w, gpu_device)
    W_hv = t["W_draft"].t().contiguous()
    _say("  inputs generated")
    path = GtoFusedPath(R=w.R, d=w.d, k=w.k, g=w.g, V=w.V, hidden=w.hidden, group_size=w.m, device=gpu_device,
                        eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=GRAD_SCALE, flags=G.GTO_FLAG_TARGET_PRUNE,
                        want_dh=True)
    path.step(t["H_cur"], t["H_ref"], t["W_draft"], t["W_target"], W_draft_hv=W_hv)
    torch.cuda.synchronize()
    n_path_rows = int((path.grad_slot >= 0).sum())
    _say(f"  GPU path done; (root, step) pairs with a gradient in the batch: {n_path_rows}")
    for tag in ("cur", "ref"):
        _properties(w, path, tag)
    # heads as fp64 in the arena, shared by all workers
    off, heads = 0, {}
    for hn in ("W_draft", "W_target"):
        heads[hn] = P.arena_put(off, t[hn].double())
        off += heads[hn]["nbytes"]
    _say("  fp64 heads in shared memory")
    rng = np.random.default_rng(5)
    n_all = w.R // w.m
    if w.w_corr > 0:     # prefer groups that carry gradient rows
        per_group = (path.grad_slot >= 0).sum(dim=1).view(n_all, w.m).sum(dim=1).cpu().numpy()
        groups = sorted(np.argsort(-per_group, kind="stable")[:n_groups].tolist())
    else:
        groups = sorted(rng.choice(n_all, size=n_groups, replace=False).tolist())
    jobs = []
    dh_slot = path.dh_slot.cpu().numpy()
    for gi in groups:
        roots = list(range(gi * w.m, (gi + 1) * w.m))
        hidden = {}
        for hn in ("H_cur", "H_ref"):
            hidden[hn] = P.arena_put(off, t[hn][roots[0]:roots[-1] + 1])
            off += hidden[hn]["nbytes"]
        dh = dict(slot=dh_slot[roots], rows={(i, s): path.dh_rows[r, s].cpu().numpy()
                                             for i, r in enumerate(roots) for s in range(w.d) if dh_slot[r, s] >= 0})
        jobs.append(dict(w=w, hidden=hidden, heads=heads, ppo=True, bundle=U.bundle_np(path, roots),
                         grad_scale=U.slice_grad_scale(GRAD_SCALE, w.m, w.R), dh=dh,
                         blas_threads=max(1, P.workers() // n_groups)))
    _say(f"  groups {groups} go to the oracle")
    results = P.run(J.fused_slice, jobs, label=name)
    tot = _collect(results, name)
    _say(f"  {name}: {tot['n_trees']} trees through the oracle ({tot['cpu_s']:.0f} CPU-s): stage 3: {tot['n_clear']} "
         f"clear of the logit error, all identical; {tot['n_ambig']} with a near tie, of which "
         f"{tot['n_same'] - tot['n_clear']} identical too; {tot['grad_rows']} gradient rows and "
         f"{tot['dh_rows']} hidden-state gradient rows compared; logit error bound E = {results[0]['E']:.2e}")
    assert tot["n_trees"] == 2 * w.m * n_groups
    # flat Gaussian logits pack the 456 candidates of a tree densely: most trees hold a pair of scores closer
    # than the worst-case budget of fp32-accumulated logits, but few of those pairs actually flip
    assert tot["n_same"] >= 0.75 * tot["n_trees"]
    if w.w_corr > 0:
        assert tot["grad_rows"] >= 8 and tot["dh_rows"] == tot["grad_rows"]
    del t, path
    torch.cuda.empty_cache()
