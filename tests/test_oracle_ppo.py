"""Pins for the group advantage (Eq. 9-10) and the clipped surrogate (Eq. 11-12), fwd and bwd."""
import math

import numpy as np
import pytest
import scipy.stats

from oracle import gto_oracle as O


def test_advantage_matches_scipy_zscore_and_identities():
    rng = np.random.default_rng(0)
    R, m = 24, 8
    rc, rr = rng.normal(3, 1, R), rng.normal(3, 1, R)
    A0 = O.group_advantage(rc, rr, m, delta=0.0)
    want = np.concatenate([scipy.stats.zscore((rc - rr)[i:i + m], ddof=0) for i in range(0, R, m)])
    np.testing.assert_allclose(A0, want, rtol=1e-12, atol=1e-13)
    delta = 1e-2
    A = O.group_advantage(rc, rr, m, delta)
    for i in range(0, R, m):
        grp = (rc - rr)[i:i + m]
        sd = grp.std()
        assert abs(A[i:i + m].mean()) < 1e-13
        np.testing.assert_allclose((A[i:i + m] ** 2).sum(), m * sd ** 2 / (sd + delta) ** 2, rtol=1e-12)
    # equal debiased rewards -> zero advantage; m = 1 -> zero advantage; no-debias variant
    assert np.all(O.group_advantage(rc, rc - 2.0, m, 1e-6) == 0.0)
    assert np.all(O.group_advantage(rc, rr, 1, 1e-6) == 0.0)
    np.testing.assert_allclose(O.group_advantage(rc, None, m, 0.0),
                               O.group_advantage(rc, np.zeros(R), m, 0.0))
    # shifting every reward of a group by a constant (position difficulty) changes nothing
    np.testing.assert_allclose(O.group_advantage(rc + 5.0, rr, m, 1e-6), O.group_advantage(rc, rr, m, 1e-6), atol=1e-12)


def _setup(seed, R=8, d=4, k=3, V=12, g=14, m=4, ref_sigma=0.2, agree=0.8):
    rng = np.random.default_rng(seed)
    D = rng.normal(0, 1.5, size=(R, d, k, V))
    Dref = D + rng.normal(0, ref_sigma, size=D.shape)
    st = O.draft_row_stats(D, k)
    sr = O.draft_row_stats(Dref, k)
    pool = O.expand_tree(st["top_tok"], st["top_logp32"], d, k)
    tree = O.select_topg(pool, g)
    T = rng.normal(0, 1.0, size=(R, d, k, V))
    for r in range(R):                       # make the target agree often so that paths are long
        for (l, j) in O.used_slots(d, k):
            if rng.random() < agree:
                T[r, l, j, st["top_tok"][r, l, j, 0]] = T[r, l, j].max() + 1.0
    ts = O.target_row_stats(T)
    path = O.accepted_path(tree, ts["t_argmax"], d)
    adv = rng.normal(0, 1, R)
    return D, Dref, st, sr, tree, path, adv, m


def test_fwd_identities():
    D, Dref, st, sr, tree, path, adv, m = _setup(1)
    R = len(adv)
    # same model on both sides: s = 1, loss_g = -mean(A_g)
    f = O.ppo_surrogate_fwd(path, tree, D, st["row_lse"], D, st["row_lse"], adv, m, 0.2)
    assert np.all(f["ratio"] == 1.0)
    np.testing.assert_allclose(f["loss_group"], [-adv[i:i + m].mean() for i in range(0, R, m)], rtol=1e-13)
    assert abs(f["loss"] - f["loss_group"].mean()) < 1e-15
    # log M equals the kept score of the last node on the path
    f = O.ppo_surrogate_fwd(path, tree, D, st["row_lse"], Dref, sr["row_lse"], adv, m, 0.2)
    for r in range(R):
        l = int(path["path_len"][r])
        if l:
            last = int(path["path_node"][r, l - 1])
            assert abs(f["logM"][r] - float(tree["sel_score"][r, last])) < 1e-4
            want = math.exp((f["logM"][r] - f["logM0"][r]) / l)
            assert abs(f["ratio"][r] - want) < 1e-14
        else:
            assert f["ratio"][r] == 1.0 and f["term"][r] == adv[r] and f["active"][r] == 0
    assert path["path_len"].max() >= 3


@pytest.mark.parametrize("shift,sign", [(+3.0, +1), (+3.0, -1), (-3.0, +1), (-3.0, -1)])
def test_clip_regions(shift, sign):
    D, Dref, st, sr, tree, path, adv, m = _setup(2)
    adv = sign * np.abs(adv)
    # a uniform shift of the reference lse moves every log ratio by `shift` per token
    f = O.ppo_surrogate_fwd(path, tree, D, st["row_lse"], D, st["row_lse"] + shift, adv, m, 0.2)
    for r in range(len(adv)):
        if path["path_len"][r] == 0:
            continue
        s = f["ratio"][r]
        assert abs(s - math.exp(shift)) < 1e-12
        if shift > 0 and sign > 0:     # s >> 1+eps, A > 0: clipped at (1+eps) A, no gradient
            assert abs(f["term"][r] - 1.2 * adv[r]) < 1e-15 and f["active"][r] == 0
        if shift > 0 and sign < 0:     # s >> 1+eps, A < 0: min picks s A (more negative), gradient flows
            assert abs(f["term"][r] - s * adv[r]) < 1e-12 and f["active"][r] == 1
        if shift < 0 and sign > 0:     # s << 1-eps, A > 0: min picks s A, gradient flows
            assert abs(f["term"][r] - s * adv[r]) < 1e-15 and f["active"][r] == 1
        if shift < 0 and sign < 0:     # s << 1-eps, A < 0: clipped at (1-eps) A
            assert abs(f["term"][r] - 0.8 * adv[r]) < 1e-15 and f["active"][r] == 0


def _loss_of(Dp, tree, path, Dref, sr, adv, m, k):
    stp = O.draft_row_stats(Dp, k)
    return O.ppo_surrogate_fwd(path, tree, Dp, stp["row_lse"], Dref, sr["row_lse"], adv, m, 0.2)["loss"]


def test_bwd_matches_central_finite_differences_and_row_sums():
    D, Dref, st, sr, tree, path, adv, m = _setup(3, R=4, d=3, k=2, V=7, g=8, m=2, ref_sigma=0.05)
    k = 2
    f = O.ppo_surrogate_fwd(path, tree, D, st["row_lse"], Dref, sr["row_lse"], adv, m, 0.2)
    gs = 0.5
    b = O.ppo_surrogate_bwd(path, tree, f, D, st["row_lse"], adv, m, gs)
    assert f["active"].sum() >= 2 and path["path_len"].max() >= 2
    h = 1e-5
    R, d, _, V = D.shape
    full = np.zeros_like(D)
    for r in range(R):
        for l in range(d):
            for j in range(k):
                for v in range(V):
                    Dp, Dm = D.copy(), D.copy()
                    Dp[r, l, j, v] += h
                    Dm[r, l, j, v] -= h
                    full[r, l, j, v] = gs * (_loss_of(Dp, tree, path, Dref, sr, adv, m, k)
                                             - _loss_of(Dm, tree, path, Dref, sr, adv, m, k)) / (2 * h)
    got = np.zeros_like(D)
    for r in range(R):
        for t in range(d):
            j = b["grad_slot"][r, t]
            if j >= 0:
                got[r, t, j] = b["grad_rows"][r, t]
    np.testing.assert_allclose(got, full, atol=2e-9)
    assert np.abs(b["grad_rows"].sum(axis=-1)).max() < 1e-14          # every row sums to zero
    for r in range(R):
        l = int(path["path_len"][r])
        assert (b["grad_slot"][r, l:] == -1).all() and not b["grad_rows"][r, l:].any()
        if not f["active"][r]:
            assert not b["grad_rows"][r].any()


def test_bwd_textbook_form_at_ratio_one():
    D, Dref, st, sr, tree, path, adv, m = _setup(4)
    f = O.ppo_surrogate_fwd(path, tree, D, st["row_lse"], D, st["row_lse"], adv, m, 0.2)
    b = O.ppo_surrogate_bwd(path, tree, f, D, st["row_lse"], adv, m, 1.0)
    R = len(adv)
    K = R // m
    for r in range(R):
        l = int(path["path_len"][r])
        for t in range(l):
            j = int(path["path_slot"][r, t])
            x = D[r, t, j]
            p = np.exp(x - x.max()); p /= p.sum()
            onehot = np.zeros_like(p); onehot[tree["sel_tok"][r, path["path_node"][r, t]]] = 1.0
            np.testing.assert_allclose(b["grad_rows"][r, t], -(adv[r] / (m * K * l)) * (onehot - p), atol=1e-15)


def test_full_path_composition_runs_and_is_consistent():
    rng = np.random.default_rng(5)
    R, d, k, V, g, m = 8, 3, 3, 30, 10, 4
    D = rng.normal(0, 2, (R, d, k, V)); T = rng.normal(0, 2, (R, d, k, V))
    Dr = D + rng.normal(0, 0.1, D.shape); Tr = rng.normal(0, 2, (R, d, k, V))
    out = O.full_path(D, T, Dr, Tr, k=k, d=d, g=g, m=m)
    np.testing.assert_allclose(out["adv"], O.group_advantage(out["cur"]["reward"]["reward_lse"],
                                                            out["ref"]["reward"]["reward_lse"], m))
    assert out["bwd"]["grad_rows"].shape == (R, d, V)


def test_token_loss_matches_scipy_entropy_kl_and_finite_differences():
    import scipy.special as sp
    rng = np.random.default_rng(8)
    R, d, k, V = 5, 2, 2, 9
    D = rng.normal(0, 1.5, (R, d, k, V)); T = rng.normal(0, 1.5, (R, d, k, V))
    out = O.token_loss(D, T)
    for r in range(R):
        pt, pm = sp.softmax(T[r, 0, 0]), sp.softmax(D[r, 0, 0])
        # H(p_T, p_M) = H(p_T) + KL(p_T || p_M)   (App. B.2)
        want = scipy.stats.entropy(pt) + scipy.stats.entropy(pt, pm)
        assert abs(out["loss_rows"][r] - want) < 1e-12
    assert abs(out["loss"] - out["loss_rows"].mean()) < 1e-15
    # same distribution: cross-entropy = entropy; one-hot target: plain negative log-likelihood
    same = O.token_loss(D, D)
    np.testing.assert_allclose(same["loss_rows"], [scipy.stats.entropy(sp.softmax(D[r, 0, 0])) for r in range(R)], rtol=1e-12)
    assert np.abs(same["grad"]).max() < 1e-16
    Th = np.full_like(T, -np.inf); tok = rng.integers(0, V, R)
    for r in range(R):
        Th[r, 0, 0, tok[r]] = 0.0
    hot = O.token_loss(D, Th)
    np.testing.assert_allclose(hot["loss_rows"], [-sp.log_softmax(D[r, 0, 0])[tok[r]] for r in range(R)], rtol=1e-12)
    # gradient: central finite differences, with a mask and a scale; only slot (0,0) matters
    w = np.array([1, 0, 1, 1, 0.0]); gs = 0.7
    ref = O.token_loss(D, T, w, gs)
    assert ref["loss_rows"][1] == 0 and not ref["grad"][1].any()
    h = 1e-6
    for r in range(R):
        for v in range(V):
            Dp, Dm = D.copy(), D.copy(); Dp[r, 0, 0, v] += h; Dm[r, 0, 0, v] -= h
            fd = gs * (O.token_loss(Dp, T, w)["loss"] - O.token_loss(Dm, T, w)["loss"]) / (2 * h)
            assert abs(fd - ref["grad"][r, v]) < 1e-8
    Dq = D.copy(); Dq[:, 1] += 3.0
    assert O.token_loss(Dq, T)["loss"] == out["loss"]
    assert np.abs(ref["grad"].sum(axis=-1)).max() < 1e-15


def test_bwd_dh_matches_central_finite_differences_through_the_lm_head():
    """The hidden-state gradient of the fused variant against finite differences of the surrogate
    taken through logits = hidden . W^T (tree, path and advantage held fixed, as in the method)."""
    rng = np.random.default_rng(11)
    R, d, k, V, Hd, g, m = 4, 3, 2, 9, 5, 8, 2
    W = rng.normal(0, 0.7, size=(V, Hd))
    H = rng.normal(0, 1.0, size=(R, d, k, Hd))
    Href = H + rng.normal(0, 0.05, size=H.shape)
    D, Dref = O.fused_logits(H, W), O.fused_logits(Href, W)
    st, sr = O.draft_row_stats(D, k), O.draft_row_stats(Dref, k)
    pool = O.expand_tree(st["top_tok"], st["top_logp32"], d, k)
    tree = O.select_topg(pool, g)
    T = rng.normal(0, 1.0, size=D.shape)
    for r in range(R):
        for (l, j) in O.used_slots(d, k):
            T[r, l, j, st["top_tok"][r, l, j, 0]] = T[r, l, j].max() + 1.0
    path = O.accepted_path(tree, O.target_row_stats(T)["t_argmax"], d)
    adv = rng.normal(0, 1, R)
    f = O.ppo_surrogate_fwd(path, tree, D, st["row_lse"], Dref, sr["row_lse"], adv, m, 0.2)
    assert f["active"].sum() >= 2 and path["path_len"].max() >= 2
    gs = 0.5
    b = O.ppo_surrogate_bwd(path, tree, f, D, st["row_lse"], adv, m, gs)
    got = O.ppo_surrogate_bwd_dh(b, W)

    def loss_of(Hp):
        Dp = O.fused_logits(Hp, W)
        return _loss_of(Dp, tree, path, Dref, sr, adv, m, k)

    h = 1e-5
    full = np.zeros_like(H)
    for idx in np.ndindex(*H.shape):
        Hp, Hm = H.copy(), H.copy()
        Hp[idx] += h
        Hm[idx] -= h
        full[idx] = gs * (loss_of(Hp) - loss_of(Hm)) / (2 * h)
    mine = np.zeros_like(H)
    for r in range(R):
        for t in range(d):
            j = b["grad_slot"][r, t]
            if j >= 0:
                mine[r, t, j] = got["dh_rows"][r, t]
    np.testing.assert_allclose(mine, full, atol=3e-9)
    assert np.abs(mine).max() > 1e-3
    assert (got["abs_bound"] >= np.abs(got["dh_rows"]) - 1e-15).all()
