"""CPU-only worker processes that run the oracle over many roots in parallel.

TEST INFRASTRUCTURE ONLY, like the oracle itself: used by the full-size parity tests and by the benchmark's
cpu_baseline leg, never by the product path.  It holds none of the method's arithmetic.

The full-size parity tests compare every root of a batch (or whole groups of it) with the oracle, which
takes about a second per root at V = 128256; fanned out over the GPU machine's host cores a whole batch takes
about a minute.  The workers are forked from the calling process BEFORE it makes its first GPU call (the
tests' conftest starts them when collection has finished, bench.py at start-up), they never touch the GPU,
and they run the oracle as it stands.

Data travels through one anonymous shared memory mapping (the "arena") created before the fork: the test
process copies a slice of the device tensors into it, the workers read it in place.  Small things (the
GPU's results for the slice, the verdict) are pickled through the pool's pipes.
"""
import mmap
import multiprocessing
import os
import sys
import time

import numpy as np

ARENA_BYTES = 24 << 30          # virtual; pages are only touched when a test writes them

_pool = None
_arena = None
_n_workers = 0


def default_workers() -> int:
    # a GPU machine gives one GPU's share of its cores (16) whatever os.cpu_count() shows; never more than that
    return max(1, min(16, os.cpu_count() or 1))


def _init_worker():
    os.environ["HIP_VISIBLE_DEVICES"] = ""       # a worker that touched the GPU by mistake would find none
    os.environ["CUDA_VISIBLE_DEVICES"] = ""
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)                     # one BLAS thread per worker; a job may raise it for itself
    except Exception:
        pass
    try:
        import torch
        torch.set_num_threads(1)
    except Exception:
        pass


def start(n_workers=None, arena_bytes=ARENA_BYTES):
    """Fork the workers.  Must run before the calling process initialises the GPU."""
    global _pool, _arena, _n_workers
    if _pool is not None:
        return
    _n_workers = n_workers or default_workers()
    _arena = mmap.mmap(-1, arena_bytes)          # MAP_SHARED | MAP_ANONYMOUS: inherited by the forked workers
    _pool = multiprocessing.get_context("fork").Pool(_n_workers, initializer=_init_worker)


def started() -> bool:
    return _pool is not None


def workers() -> int:
    return _n_workers


def stop():
    global _pool, _arena
    if _pool is not None:
        _pool.terminate()
        _pool.join()
        _pool = None
    _arena = None


def arena_np(offset: int, shape, dtype) -> np.ndarray:
    """A view of the arena (same bytes in the test process and in every worker)."""
    n = int(np.prod(shape))
    return np.frombuffer(_arena, dtype=dtype, count=n, offset=offset).reshape(shape)


def arena_put(offset: int, tensor) -> dict:
    """Copy a device (or host) torch tensor into the arena at `offset`; returns the handle a job carries.
    bf16 travels as its 16-bit patterns."""
    import torch
    t = tensor.contiguous()
    kind = {torch.bfloat16: "bf16", torch.float32: "f32", torch.float64: "f64"}[t.dtype]
    if kind == "bf16":
        t = t.view(torch.int16)
    nbytes = t.numel() * t.element_size()
    assert offset % 256 == 0 and offset + nbytes <= len(_arena), "arena too small for this slice"
    dst = torch.frombuffer(_arena, dtype=t.dtype, count=t.numel(), offset=offset).view(t.shape)
    dst.copy_(t)
    return {"offset": offset, "shape": tuple(t.shape), "kind": kind, "nbytes": (nbytes + 255) & ~255}


def arena_get(handle, rows=None) -> np.ndarray:
    """The array behind a handle, as fp32 (bf16 / f32 handles) or fp64; `rows` = slice of the first axis."""
    kind = handle["kind"]
    dt = {"bf16": np.uint16, "f32": np.float32, "f64": np.float64}[kind]
    a = arena_np(handle["offset"], handle["shape"], dt)
    if rows is not None:
        a = a[rows]
    if kind == "bf16":                            # bf16 -> fp32 is exact: the pattern is the upper half
        return (a.astype(np.uint32) << 16).view(np.float32)
    return a


def run(func, jobs, label="", quiet=False):
    """Run func(job) for every job on the workers; results in job order.  Prints one line per finished job
    (the work's own progress): to stdout, or to stderr when `quiet` (a caller whose stdout is its result)."""
    t0 = time.time()
    pending = [_pool.apply_async(func, (job,)) for job in jobs]
    out = []
    for i, p in enumerate(pending):
        out.append(p.get())
        print(f"    {label} job {i + 1}/{len(jobs)} done at {time.time() - t0:.1f} s", flush=True,
              file=sys.stderr if quiet else sys.stdout)
    return out


def timed_full_path(job):
    """Worker job of the benchmark's cpu_baseline leg: the oracle's whole path (both trees, rewards, advantage,
    surrogate, gradient; or build + reward + walk of one tree for a reward-only workload) over the roots
    whose logits sit in the arena.  Returns the seconds it took, the trees it scored and, from the oracle's
    near-tie audit, how many of them hold a ranking decision within fp32 rounding (several results correct).
    job: logits {name: handle}, V, k, d, g, m, eta, eps, delta, full_path; for the fused workload instead
    hidden {H_cur, H_ref} and heads {W_draft, W_target} (fp64)."""
    from oracle import gto_oracle as O
    t0 = time.time()
    k, d, g = job["k"], job["d"], job["g"]
    if "hidden" in job:
        H = {n: arena_get(h) for n, h in job["hidden"].items()}
        Wd, Wt = arena_get(job["heads"]["W_draft"]), arena_get(job["heads"]["W_target"])
        L = {"D_cur": O.fused_logits(H["H_cur"], Wd), "T_cur": O.fused_logits(H["H_cur"], Wt),
             "D_ref": O.fused_logits(H["H_ref"], Wd), "T_ref": O.fused_logits(H["H_ref"], Wt)}
        # the other side accumulates these logits in fp32: the audit is told by how much they may differ
        job = dict(job, logit_err=O.fp32_accumulation_error(Wd.shape[1], max(float(np.abs(v).max()) for v in L.values())))
    else:
        L = {n: arena_get(h)[..., :job["V"]] for n, h in job["logits"].items()}
    n = L["D_cur"].shape[0]
    if job["full_path"]:
        out = O.full_path(L["D_cur"], L["T_cur"], L["D_ref"], L["T_ref"], k=k, d=d, g=g, m=job["m"], eta=job["eta"],
                          eps=job["eps"], delta=job["delta"], grad_scale=0.5, logit_err=job.get("logit_err", 0.0))
        margins = [np.minimum(out[t]["pool"]["min_margin"], out[t]["tree"]["min_margin"]) for t in ("cur", "ref")]
        trees = 2 * n
    else:
        ds = O.draft_row_stats(L["D_cur"], k)
        pool = O.expand_tree(ds["top_tok"], ds["top_logp32"], d, k, ds["top_logp64"], ds["top_logit"])
        tree = O.select_topg(pool, g, audit=True)
        ts = O.target_row_stats(L["T_cur"])
        O.tree_reward(tree, L["T_cur"], ts["t_lse"], job["eta"])
        O.accepted_path(tree, ts["t_argmax"], d)
        margins = [np.minimum(pool["min_margin"], tree["min_margin"])]
        trees = n
    near = int(sum((mg < 1.0).sum() for mg in margins))
    return dict(seconds=time.time() - t0, trees=trees, near_ties=near)
