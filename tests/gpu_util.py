"""Helpers for the GPU parity tests: run the HIP path, fetch results, compare with the oracle."""
import math

import numpy as np
import torch

from oracle import gto_oracle as O

TAU = 1.0           # oracle's gap-to-error-budget ratio below which a ranking decision is a near tie


def alloc_poisoned(alloc, cfg, device):
    """Output buffers filled with a poison pattern instead of zeros: an entry the kernels should have
    written but did not, or a read of one they never wrote, then shows up as a wild value."""
    out = alloc(cfg, device)
    for t in out.values():
        if t.dtype == torch.int32:
            t.fill_(0x7F7F7F7F)
        else:
            t.fill_(float("nan"))
    return out


def poison_path(path):
    """Poison every output buffer of a GtoPath / GtoFusedPath (see alloc_poisoned)."""
    for tag in path.buf:
        for grp in path.buf[tag].values():
            for t in grp.values():
                t.fill_(0x7F7F7F7F if t.dtype == torch.int32 else float("nan"))
    for t in path.ppo.values():
        t.fill_(0x7F7F7F7F if t.dtype == torch.int32 else float("nan"))
    path.adv.fill_(float("nan"))


def to_np(d):
    return {k: v.detach().cpu().numpy() for k, v in d.items() if v is not None}


def logits_np(t) -> np.ndarray:
    """The exact values the GPU sees, as float32 (bf16 -> fp32 is exact); numpy arrays pass through."""
    if isinstance(t, np.ndarray):
        return t
    return t.detach().float().cpu().numpy()


def used_mask(R, d, k):
    m = np.zeros((R, d, k), dtype=bool)
    m[:, 0, 0] = True
    m[:, 1:, :] = True
    return m


def check_row_stats(gd, od, D_np, k, lse_rtol=1e-6):
    """Stage 1 (draft rows): ids and max exact, lse and logp within tolerance."""
    R, d, kk, V = D_np.shape
    m = used_mask(R, d, kk)
    assert np.array_equal(gd["top_tok"][m], od["top_tok"][m]), "top-k token ids differ"
    assert np.array_equal(gd["row_max"][m], od["row_max"][m].astype(np.float32)), "row max differs"
    np.testing.assert_allclose(gd["row_lse"][m], od["row_lse"][m], rtol=lse_rtol, atol=1e-6)
    a, b = gd["top_logp"][m].astype(np.float64), od["top_logp64"][m]
    fin = np.isfinite(b)
    assert np.array_equal(np.isfinite(a), fin)
    # logp = logit - lse: one fp32 rounding of a number of size |logp| plus the lse error
    assert np.all(np.abs(a[fin] - b[fin]) <= 1.5e-6 * np.maximum(1.0, np.abs(b[fin]))), \
        float(np.max(np.abs(a[fin] - b[fin])))


def check_target_stats(gt, ot, lse_rtol=1e-6, need=None):
    """`need` ([R, d, k] flags): with target-row pruning only the slots whose node has a kept child are
    streamed; the others keep whatever the buffer held."""
    R, d, k = ot["t_argmax"].shape
    m = used_mask(R, d, k)
    if need is not None:
        m = m & (need != 0)
    assert np.array_equal(gt["t_argmax"][m], ot["t_argmax"][m]), "target argmax differs"
    assert np.array_equal(gt["t_max"][m], ot["t_max"][m].astype(np.float32))
    np.testing.assert_allclose(gt["t_lse"][m], ot["t_lse"][m], rtol=lse_rtol, atol=1e-6)


INT_POOL = ("cand_tok", "cand_parent", "cand_depth", "cand_pslot", "cand_slot", "slot_cand")
INT_TREE = ("sel_cand", "sel_tok", "sel_parent", "sel_depth", "sel_pslot", "sel_slot", "sel_leaf", "n_sel", "slot_need")
INT_PATH = ("path_len", "path_node", "path_slot")


def oracle_from_gpu_stats(gd, gt, T_np, d, k, g, eta):
    """Stage 2 reference: the oracle's integer logic fed the GPU's own fp32 row statistics."""
    pool = O.expand_tree(gd["top_tok"], gd["top_logp"], d, k)
    tree = O.select_topg(pool, g)
    rew = O.tree_reward(tree, T_np, gt["t_lse"].astype(np.float64), eta)
    path = O.accepted_path(tree, gt["t_argmax"], d)
    return pool, tree, rew, path


def _scores_equal(a, b, exact, atol=4e-6):
    if exact:
        return np.array_equal(a, b)
    fin = np.isfinite(b)
    return np.array_equal(np.isfinite(a), fin) and \
        np.all(np.abs(a[fin].astype(np.float64) - b[fin]) <= 1e-6 * np.abs(b[fin]) + atol)


def check_stage2(gpool, gtree, grew, opool, otree, orew, opath, roots=None, exact_scores=True, rtol=1e-5,
                 score_atol=4e-6):
    """Every integer output bit-exact.  Scores: bit-exact when both sides started from the same fp32
    row statistics (stage 2); within a few fp32 roundings against the pure fp64 oracle (stage 3)."""
    sl = slice(None) if roots is None else roots
    for name in INT_POOL:
        assert np.array_equal(gpool[name][sl], opool[name][sl]), name
    assert _scores_equal(gpool["cand_score"][sl], opool["cand_score"][sl], exact_scores, score_atol), "cand_score"
    for name in INT_TREE:
        assert np.array_equal(gtree[name][sl], otree[name][sl]), name
    assert _scores_equal(gtree["sel_score"][sl], otree["sel_score"][sl], exact_scores, score_atol), "sel_score"
    for name in INT_PATH:
        assert np.array_equal(grew[name][sl], opath[name][sl]), name
    assert np.array_equal(grew["n_leaves"][sl], orew["n_leaves"][sl])
    check_reward_floats(grew, orew, roots, rtol=rtol)


def same_integers(gpool, gtree, grew, opool, otree, orew, opath):
    """Per root: do all integer outputs (pool, kept tree, walk, leaf count) agree?  [n] bool."""
    n = gtree["n_sel"].shape[0]
    ok = np.ones(n, dtype=bool)
    for names, a, b in ((INT_POOL, gpool, opool), (INT_TREE, gtree, otree), (INT_PATH, grew, opath),
                        (("n_leaves",), grew, orew)):
        for name in names:
            ok &= (a[name].reshape(n, -1) == b[name].reshape(n, -1)).all(axis=1)
    return ok


def stage3(b, o, clear_mask, **kw):
    """End to end against the pure fp64 oracle.  Roots whose ranking decisions are all clear of rounding
    (`clear_mask`) must match exactly.  A root with a near tie may legitimately differ; when it does not, its
    floats are held to the same tolerances.  Returns (clear roots, roots identical end to end)."""
    clear = np.nonzero(clear_mask)[0]
    check_stage2(b["pool"], b["tree"], b["reward"], o["pool"], o["tree"], o["reward"], o["path"], roots=clear,
                 exact_scores=False, **kw)
    same = same_integers(b["pool"], b["tree"], b["reward"], o["pool"], o["tree"], o["reward"], o["path"])
    assert same[clear].all()
    lucky = np.nonzero(same & ~clear_mask)[0]
    check_stage2(b["pool"], b["tree"], b["reward"], o["pool"], o["tree"], o["reward"], o["path"], roots=lucky,
                 exact_scores=False, **kw)
    return len(clear), int(same.sum())


def check_reward_floats(grew, orew, roots=None, rtol=1e-5):
    sl = slice(None) if roots is None else roots
    np.testing.assert_allclose(grew["node_q"][sl], orew["node_q"][sl], rtol=rtol, atol=1e-30)
    np.testing.assert_allclose(grew["node_cum"][sl], orew["node_cum"][sl], rtol=rtol, atol=1e-30)
    for i, key in enumerate(("reward_lse", "reward_max", "reward_mean", "reward_nodesum")):
        np.testing.assert_allclose(grew["reward_aux"][sl][:, i], orew[key][sl], rtol=rtol, atol=1e-30, err_msg=key)


# ------------------------------------------------------------------------------------------------
# Comparisons on host copies ("bundles") of the GPU's outputs.  They take numpy only, so that the same
# code runs in the test process (small cases) and in the CPU-only oracle workers (full-size cases).
GROUPS = ("dstats", "tstats", "pool", "tree", "reward")


def bundle_np(path, roots=None, with_ppo=True, grad="rows"):
    """Host copy of every output of a GtoPath / GtoFusedPath for the roots in `roots` (default all).
    grad: "rows" = gradient rows as {(i, t): row} for the rows that carry a gradient (i = position in
    `roots`), "dense" = the whole [n, d, V] array, None = no gradient."""
    n_all = path.cfg.R
    roots = list(range(n_all)) if roots is None else list(roots)
    idx = torch.as_tensor(roots, device=path.adv.device if hasattr(path, "adv") else None, dtype=torch.long)
    out = {"roots": roots, "pruned": bool(path.cfg.flags & 2)}
    for tag in path.buf:
        out[tag] = {grp: {k: v[idx].cpu().numpy() for k, v in path.buf[tag][grp].items()
                          if v is not None and k != "accept_u"} for grp in GROUPS}
    if with_ppo and hasattr(path, "ppo"):
        m = path.cfg.group_size
        out["adv"] = path.adv[idx].cpu().numpy()
        out["ppo"] = {k: v[idx].cpu().numpy() for k, v in path.ppo.items() if k not in ("loss_group", "loss")}
        lg = path.ppo["loss_group"].cpu().numpy()
        out["ppo"]["loss_group_of_root"] = lg[np.asarray(roots) // m]
        out["ppo"]["loss"] = path.ppo["loss"].cpu().numpy()
        if grad is not None and getattr(path, "want_grad", False):
            slot = path.grad_slot[idx].cpu().numpy()
            out["grad_slot"] = slot
            if grad == "dense":
                out["grad_rows"] = path.grad_rows[idx].cpu().numpy()
            else:
                out["grad_rows"] = {(i, t): path.grad_rows[roots[i], t].cpu().numpy()
                                    for i in range(len(roots)) for t in range(slot.shape[1]) if slot[i, t] >= 0}
    return out


def compare_trees(w, sub, bundle, ora=None):
    """Stages 1-3 of the streaming path for the roots of `bundle` (`sub` holds their logits, fp32 numpy,
    already cut to the vocabulary).  Returns (oracle results, near-tie trees, clear trees, trees identical to
    the pure oracle's end to end)."""
    if ora is None:
        ora = O.full_path(sub["D_cur"], sub["T_cur"], sub.get("D_ref", sub["D_cur"]), sub.get("T_ref", sub["T_cur"]),
                          k=w.k, d=w.d, g=w.g, m=1, eta=w.eta, eps=w.eps, delta=w.delta, want_grad=False)
    n = sub["D_cur"].shape[0]
    n_ambig = n_clear = n_same = 0
    for tag in (("cur", "ref") if w.full_path else ("cur",)):
        b, o = bundle[tag], ora[tag]
        Dn, Tn = sub.get("D_" + tag, sub["D_cur"]), sub.get("T_" + tag, sub["T_cur"])
        check_row_stats(b["dstats"], o["dstats"], Dn, w.k)                       # stage 1
        check_target_stats(b["tstats"], o["tstats"], need=b["tree"]["slot_need"] if bundle.get("pruned") else None)
        pool2, tree2, rew2, path2 = oracle_from_gpu_stats(b["dstats"], b["tstats"], Tn, w.d, w.k, w.g, w.eta)
        check_stage2(b["pool"], b["tree"], b["reward"], pool2, tree2, rew2, path2)     # stage 2
        margin = np.minimum(o["pool"]["min_margin"], o["tree"]["min_margin"])
        nc, ns = stage3(b, o, margin >= TAU)                                      # stage 3
        n_ambig += n - nc
        n_clear += nc
        n_same += ns
    return ora, n_ambig, n_clear, n_same


def _grad_row(grad_rows, i, t):
    return grad_rows[(i, t)] if isinstance(grad_rows, dict) else grad_rows[i, t]


def compare_ppo(w, sub, bundle, ora, grad_scale=0.5, reward_key="reward_lse", zero_fill=False, untouched=None, E=0.0):
    """Advantage, surrogate and gradient of whole groups: the roots of `bundle` are consecutive groups of
    w.m roots and `ora` is O.full_path over exactly these roots with m = w.m and the same grad_scale
    (scaled by the caller when the batch has more groups than the slice, see slice_grad_scale).
    (a) the kernels on the GPU's own inputs: oracle arithmetic fed the GPU's rewards / trees / statistics;
    (b) end to end against the pure fp64 oracle where the trees agree.
    E: absolute error of the GPU's logits against `sub` (0 for stored logits; the fused variant's fp32
    accumulation error, see logit_error_bound); it widens the float tolerances: a log-probability is then off
    by up to 2 E (logit and log-sum-exp), a sum over a path by 2 d E.
    Returns (whether (b) ran, gradient rows compared, the oracle's group losses on the GPU's inputs)."""
    rt = 1e-5 + 4 * E
    cur, ref = bundle["cur"], bundle["ref"]
    g_tree, g_rew = cur["tree"], cur["reward"]
    same_tree = all(np.array_equal(g_tree[n], ora["cur"]["tree"][n]) for n in INT_TREE) and \
        all(np.array_equal(g_rew[n], ora["cur"]["path"][n]) for n in INT_PATH) and \
        np.array_equal(ref["tree"]["sel_cand"], ora["ref"]["tree"]["sel_cand"])
    g_adv = bundle["adv"]
    adv_same_in = O.group_advantage(g_rew["reward"].astype(np.float64), ref["reward"]["reward"].astype(np.float64),
                                    w.m, w.delta)
    np.testing.assert_allclose(g_adv, adv_same_in, rtol=2e-6, atol=1e-6)
    gd, gr = cur["dstats"], ref["dstats"]
    gpath = {n: g_rew[n] for n in INT_PATH}
    f2 = O.ppo_surrogate_fwd(gpath, g_tree, sub["D_cur"], gd["row_lse"].astype(np.float64), sub["D_ref"],
                             gr["row_lse"].astype(np.float64), g_adv.astype(np.float64), w.m, w.eps)
    gp = bundle["ppo"]
    for n in ("logM", "logM0", "ratio", "term"):
        np.testing.assert_allclose(gp[n], f2[n], rtol=rt, atol=1e-6 + 2 * w.d * E, err_msg=n)
    if E == 0.0:
        assert np.array_equal(gp["active"], f2["active"])
    else:       # a ratio within the logit error of a clip boundary may fall on either side
        edge = np.minimum(np.abs(f2["ratio"] - (1 - w.eps)), np.abs(f2["ratio"] - (1 + w.eps))) <= 8 * E
        assert np.array_equal(gp["active"][~edge], f2["active"][~edge])
        f2["active"], f2["ratio"] = gp["active"].copy(), gp["ratio"].astype(np.float64)
    np.testing.assert_allclose(gp["loss_group_of_root"], np.repeat(f2["loss_group"], w.m), rtol=rt,
                               atol=1e-6 + 2 * w.d * E)
    # gradient rows against the oracle's own fp64 softmax (same path, advantage and ratio)
    b2 = O.ppo_surrogate_bwd(gpath, g_tree, f2, sub["D_cur"], ora["cur"]["dstats"]["row_lse"],
                             g_adv.astype(np.float64), w.m, grad_scale)
    np.testing.assert_allclose(gp["coef"], b2["coef"], rtol=rt, atol=1e-12)
    n_rows = 0
    if "grad_slot" in bundle:
        g_slot, g_rows = bundle["grad_slot"], bundle["grad_rows"]
        want_slot = np.where((b2["coef"] != 0)[:, None], b2["grad_slot"], -1)
        assert np.array_equal(g_slot, want_slot)
        for i in range(g_slot.shape[0]):
            for t in range(w.d):
                if g_slot[i, t] >= 0:
                    ref_row = b2["grad_rows"][i, t]
                    scale = np.abs(ref_row).max()
                    assert np.abs(_grad_row(g_rows, i, t) - ref_row).max() <= rt * scale + 1e-12, (i, t)
                    n_rows += 1
                elif isinstance(g_rows, np.ndarray):
                    if zero_fill:
                        assert not g_rows[i, t].any()
                    elif untouched is not None:
                        assert (g_rows[i, t] == untouched).all()
    if same_tree:
        key = reward_key
        sd = np.array([np.std((ora["cur"]["reward"][key] - ora["ref"]["reward"][key])[i:i + w.m])
                       for i in range(0, len(g_adv), w.m)]).repeat(w.m)
        # standardisation divides the rewards' error (fp32 rounding, plus 4 d E relative for the fused variant)
        # by the group's spread
        rew_err = 4e-6 + 4 * w.d * E * float(np.abs(ora["cur"]["reward"][key]).max())
        tol = rt * (1 + np.abs(ora["adv"])) + rew_err * (1 + np.abs(ora["adv"])) / (sd + w.delta)
        assert np.all(np.abs(g_adv - ora["adv"]) <= tol)
        ok = sd > 0.05 + 1e4 * E     # groups whose spread is far above the reward error
        np.testing.assert_allclose(gp["ratio"], ora["ppo"]["ratio"], rtol=rt)
        # the term of Eq. 12 is (clipped) ratio x advantage: it inherits the advantage's error bound times the
        # ratio, plus the relative error of the ratio itself
        o_term, o_ratio = ora["ppo"]["term"], np.abs(ora["ppo"]["ratio"])
        term_tol = np.maximum(o_ratio, 1 + w.eps) * tol + (2e-4 + 100 * E) * np.abs(o_term) + 1e-7
        assert np.all(np.abs(gp["term"] - o_term)[ok] <= term_tol[ok]), \
            float(np.max((np.abs(gp["term"] - o_term) / term_tol)[ok]))
    return same_tree, n_rows, f2["loss_group"]


def slice_grad_scale(grad_scale, n_slice_roots, n_batch_roots):
    """The gradient coefficient carries 1 / (m K) with K the number of groups of the BATCH; an oracle call
    over a slice of whole groups sees K_slice instead.  The coefficient is linear in grad_scale, so the
    slice's call gets grad_scale * K_slice / K_batch."""
    return grad_scale * n_slice_roots / n_batch_roots


# ------------------------------------------------------------------------------------------------ fused variant
logit_error_bound = O.fp32_accumulation_error      # E: see the oracle for the derivation


def compare_trees_fused(w, L, bundle, ora=None, E=None):
    """Stages 1-3 of the fused LM-head variant.  `L` holds the oracle's fp64 logits (O.fused_logits) of the
    bundle's roots.  The GPU accumulates its logits in fp32, so every logit carries an absolute error of up
    to E; row top-k / argmax are compared where the oracle's row margins are clear of E, tree decisions
    where the oracle's audit (with E in its budget) says so, floats within max(1e-5, 4 d E) relative.
    Returns (oracle results, E, near-tie trees, clear trees, trees identical to the pure oracle's end to end)."""
    if E is None:
        E = logit_error_bound(w.hidden, max(float(np.abs(v).max()) for v in L.values()))
    rtol = max(1e-5, 4 * w.d * E)
    if ora is None:
        ora = O.full_path(L["D_cur"], L["T_cur"], L["D_ref"], L["T_ref"], k=w.k, d=w.d, g=w.g, m=1, eta=w.eta,
                          eps=w.eps, delta=w.delta, want_grad=False, logit_err=E)
    n = L["D_cur"].shape[0]
    n_ambig = n_clear = n_same = 0
    m = used_mask(n, w.d, w.k)
    for tag in ("cur", "ref"):
        b = bundle[tag]
        gd, gt = b["dstats"], b["tstats"]
        o, Dn, Tn = ora[tag], L["D_" + tag], L["T_" + tag]
        mt = m & (b["tree"]["slot_need"] != 0) if bundle.get("pruned") else m
        # stage 1: the GPU's logits at its own top tokens are the oracle's within E; statistics within E
        g_logit = gd["top_logp"].astype(np.float64) + gd["row_lse"].astype(np.float64)[..., None]
        o_at = np.take_along_axis(Dn, gd["top_tok"].astype(np.int64).clip(0, w.V - 1), axis=-1)
        assert np.abs(g_logit - o_at)[m].max() <= E + 4e-6, float(np.abs(g_logit - o_at)[m].max())
        assert np.abs(gd["row_lse"] - o["dstats"]["row_lse"])[m].max() <= E + 2e-6
        assert np.abs(gt["t_lse"] - o["tstats"]["t_lse"])[mt].max() <= E + 2e-6
        assert np.abs(gd["row_max"] - o["dstats"]["row_max"])[m].max() <= E
        rm_d, rm_t = O.row_margins(Dn, w.k, E), O.row_margins(Tn, 1, E)
        clear_rows = (rm_d >= 1.0) & (rm_t >= 1.0)
        for r in np.nonzero(clear_rows)[0]:
            assert np.array_equal(gd["top_tok"][r][m[r]], o["dstats"]["top_tok"][r][m[r]]), (tag, r)
            assert np.array_equal(gt["t_argmax"][r][mt[r]], o["tstats"]["t_argmax"][r][mt[r]]), (tag, r)
        # stage 2: oracle logic on the GPU's own statistics, bit for bit
        pool2, tree2, rew2, path2 = oracle_from_gpu_stats(gd, gt, Tn, w.d, w.k, w.g, w.eta)
        check_stage2(b["pool"], b["tree"], b["reward"], pool2, tree2, rew2, path2, rtol=rtol)
        # stage 3: end to end where every decision is clear of the logit error
        margin = np.minimum(o["pool"]["min_margin"], o["tree"]["min_margin"])
        nc, ns = stage3(b, o, (margin >= 1.0) & clear_rows, rtol=rtol, score_atol=4e-6 + 2 * w.d * E)
        n_ambig += n - nc
        n_clear += nc
        n_same += ns
    return ora, E, n_ambig, n_clear, n_same


def compare_dh(w, L, bundle, dh, W64, grad_scale, E, row_lse):
    """Hidden-state gradient rows of the fused backward against the oracle's fp64 contraction, on the GPU's
    own tree, path, advantage and ratio.  Tolerance: the gradient row is staged as hi + lo bf16 (2^-17
    relative per entry), built from fp32 logits (error E) and summed in fp32, all relative to
    sum_v |G| |W| (the oracle's abs_bound).  `row_lse`: the oracle's fp64 log-sum-exps of the current draft
    rows.  Returns the number of rows compared."""
    cur = bundle["cur"]
    g_tree, g_rew, gp = cur["tree"], cur["reward"], bundle["ppo"]
    gpath = {n: g_rew[n] for n in INT_PATH}
    f2 = dict(active=gp["active"], ratio=gp["ratio"].astype(np.float64))
    b2 = O.ppo_surrogate_bwd(gpath, g_tree, f2, L["D_cur"], row_lse, bundle["adv"].astype(np.float64), w.m,
                             grad_scale)
    want = O.ppo_surrogate_bwd_dh(b2, W64)
    slot = dh["slot"]
    assert np.array_equal(slot, np.where((b2["coef"] != 0)[:, None], b2["grad_slot"], -1))
    n = 0
    for (i, t), got in dh["rows"].items():
        assert slot[i, t] >= 0
        tol = (2.0 ** -17 + 2 * E + 1e-6) * want["abs_bound"][i, t] + 1e-30
        err = np.abs(got - want["dh_rows"][i, t])
        assert (err <= tol).all(), (i, t, float((err / tol).max()))
        n += 1
    assert n == int((slot >= 0).sum())
    return n
