"""Jobs the CPU-only oracle workers run (see oracle/pool.py): the oracle over one slice of roots, compared
with the GPU's results for that slice.  A job returns a small verdict; it never raises (a failure comes
back as text, so that the test process can report the slice and go on to read the other verdicts)."""
import time
import traceback

import numpy as np

import gpu_util as U
from oracle import pool as P
from oracle import gto_oracle as O


def _verdict(job, fn):
    t0 = time.time()
    try:
        out = fn()
        out.update(ok=True)
    except Exception:
        out = dict(ok=False, err=traceback.format_exc())
    out.update(roots=(job["bundle"]["roots"][0], job["bundle"]["roots"][-1]), seconds=time.time() - t0)
    return out


def streaming_slice(job):
    """Stored-logits path.  job: w (workload), V, logits {name: arena handle of the whole resident slice},
    rows (slice of that slice's first axis), bundle (GPU results of these roots), ppo (bool: the roots are
    whole groups and the bundle carries advantage / surrogate / gradient), grad_scale (already scaled to
    the slice), reward_key."""
    def body():
        w, V = job["w"], job["V"]
        sub = {n: P.arena_get(h, job["rows"])[..., :V] for n, h in job["logits"].items()}
        if job.get("ppo"):
            ora = O.full_path(sub["D_cur"], sub["T_cur"], sub["D_ref"], sub["T_ref"], k=w.k, d=w.d, g=w.g, m=w.m,
                              eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=job["grad_scale"])
        else:
            ora = None
        ora, n_ambig, n_clear, n_same = U.compare_trees(w, sub, job["bundle"], ora)
        out = dict(n_trees=(2 if w.full_path else 1) * sub["D_cur"].shape[0], n_ambig=n_ambig, n_clear=n_clear,
                   n_same=n_same)
        if job.get("ppo"):
            e2e, n_rows, loss_group = U.compare_ppo(w, sub, job["bundle"], ora, grad_scale=job["grad_scale"],
                                                    reward_key=job.get("reward_key", "reward_lse"))
            out.update(ppo_e2e=bool(e2e), grad_rows=n_rows, loss_group=loss_group,
                       path_rows=int(job["bundle"]["cur"]["reward"]["path_len"].sum()))
        return out
    return _verdict(job, body)


def fused_slice(job):
    """Fused LM-head path.  job: w (fused workload), hidden {H_cur, H_ref: arena handles of the hidden states
    of the bundle's roots}, heads {W_draft, W_target: arena handles of the fp64 heads [V, hidden]}, bundle,
    ppo, grad_scale, blas_threads, dh (optional: {"rows": {(i, t): dh row}, "slot": [n, d]})."""
    def body():
        w = job["w"]
        try:
            from threadpoolctl import threadpool_limits
            limiter = threadpool_limits(job.get("blas_threads", 1))
        except Exception:
            limiter = None
        H = {n: P.arena_get(h) for n, h in job["hidden"].items()}
        Wd, Wt = P.arena_get(job["heads"]["W_draft"]), P.arena_get(job["heads"]["W_target"])
        L = {"D_cur": O.fused_logits(H["H_cur"], Wd), "T_cur": O.fused_logits(H["H_cur"], Wt),
             "D_ref": O.fused_logits(H["H_ref"], Wd), "T_ref": O.fused_logits(H["H_ref"], Wt)}
        E = U.logit_error_bound(w.hidden, max(float(np.abs(v).max()) for v in L.values()))
        ora = O.full_path(L["D_cur"], L["T_cur"], L["D_ref"], L["T_ref"], k=w.k, d=w.d, g=w.g,
                          m=w.m if job.get("ppo") else 1, eta=w.eta, eps=w.eps, delta=w.delta,
                          grad_scale=job.get("grad_scale", 1.0), want_grad=bool(job.get("ppo")), logit_err=E)
        ora, E, n_ambig, n_clear, n_same = U.compare_trees_fused(w, L, job["bundle"], ora=ora, E=E)
        out = dict(n_trees=2 * L["D_cur"].shape[0], n_ambig=n_ambig, n_clear=n_clear, n_same=n_same, E=E)
        if job.get("ppo"):
            e2e, n_rows, loss_group = U.compare_ppo(w, L, job["bundle"], ora, grad_scale=job["grad_scale"], E=E)
            out.update(ppo_e2e=bool(e2e), grad_rows=n_rows, loss_group=loss_group,
                       path_rows=int(job["bundle"]["cur"]["reward"]["path_len"].sum()))
            if job.get("dh") is not None:
                out.update(dh_rows=U.compare_dh(w, L, job["bundle"], job["dh"], Wd, job["grad_scale"], E,
                                                ora["cur"]["dstats"]["row_lse"]))
        if limiter is not None:
            limiter.restore_original_limits()
        return out
    return _verdict(job, body)
