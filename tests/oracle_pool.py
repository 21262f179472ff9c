"""CPU-only worker processes that run the oracle over many roots in parallel.

The full-size parity tests compare every root of a batch (or whole groups of it) with the oracle, which
takes about a second per root at V = 128256; fanned out over the GPU machine's host cores a whole batch takes
about a minute.  The workers are forked from the test process BEFORE it makes its first GPU call (conftest
starts them when collection has finished), they never touch the GPU, and they run the oracle as it stands.

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


def run(func, jobs, label=""):
    """Run func(job) for every job on the workers; results in job order.  Prints one line per finished job
    (the work's own progress)."""
    t0 = time.time()
    pending = [_pool.apply_async(func, (job,)) for job in jobs]
    out = []
    for i, p in enumerate(pending):
        out.append(p.get())
        print(f"    {label} job {i + 1}/{len(jobs)} done at {time.time() - t0:.1f} s", flush=True)
    sys.stdout.flush()
    return out
