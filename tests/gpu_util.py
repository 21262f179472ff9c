"""Helpers for the GPU parity tests: run the HIP path, fetch results, compare with the oracle."""
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


def check_target_stats(gt, ot, lse_rtol=1e-6):
    R, d, k = ot["t_argmax"].shape
    m = used_mask(R, d, k)
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


def check_reward_floats(grew, orew, roots=None, rtol=1e-5):
    sl = slice(None) if roots is None else roots
    np.testing.assert_allclose(grew["node_q"][sl], orew["node_q"][sl], rtol=rtol, atol=1e-30)
    np.testing.assert_allclose(grew["node_cum"][sl], orew["node_cum"][sl], rtol=rtol, atol=1e-30)
    for i, key in enumerate(("reward_lse", "reward_max", "reward_mean", "reward_nodesum")):
        np.testing.assert_allclose(grew["reward_aux"][sl][:, i], orew[key][sl], rtol=rtol, atol=1e-30, err_msg=key)
