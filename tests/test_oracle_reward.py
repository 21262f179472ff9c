"""Pins for the Draft Tree Reward (Eq. 2-5, ablation aggregates, App. A) and the greedy walk."""
import math

import numpy as np
import pytest
import scipy.special as sp

import brute
from oracle import gto_oracle as O


def _case(seed, R, d, k, V, g, sigma=1.5):
    rng = np.random.default_rng(seed)
    D = rng.normal(0, sigma, size=(R, d, k, V))
    T = rng.normal(0, sigma, size=(R, d, k, V))
    st = O.draft_row_stats(D, k)
    pool = O.expand_tree(st["top_tok"], st["top_logp32"], d, k, st["top_logp64"], st["top_logit"])
    tree = O.select_topg(pool, g)
    ts = O.target_row_stats(T)
    return D, T, pool, tree, ts


@pytest.mark.parametrize("seed,V,k,d,g", [(0, 4, 2, 3, 6), (1, 4, 3, 3, 12), (2, 5, 2, 3, 4), (3, 4, 2, 2, 6)])
def test_nodesum_equals_enumeration_of_all_rollouts(seed, V, k, d, g):
    D, T, pool, tree, ts = _case(seed, 2, d, k, V, g)
    rew = O.tree_reward(tree, T, ts["t_lse"], 1.0)
    for r in range(2):
        kept, expanded = brute.build_tree(D[r], k, d, g)
        paths = [p for p, _ in kept]
        e_enum = brute.expected_accept_len_enumerate(paths, expanded, T[r], d)
        e_rec = brute.expected_accept_len_recursive(paths, expanded, T[r])
        assert abs(rew["reward_nodesum"][r] - e_enum) < 1e-12
        assert abs(rew["reward_nodesum"][r] - e_rec) < 1e-12
        # per-sequence expected acceptance lengths (Eq. 3-4) and their aggregates (Eq. 5, ablation)
        Ls = brute.sequence_lengths(paths, expanded, T[r])
        opaths = brute.oracle_paths(pool, tree, r)
        got = {opaths[i]: rew["node_cum"][r, i] for i in range(int(tree["n_sel"][r])) if tree["sel_leaf"][r, i]}
        assert set(got) == set(Ls)
        for p in Ls:
            assert abs(got[p] - Ls[p]) < 1e-12
        vals = np.array(list(Ls.values()))
        for eta in (1.0, 0.25, 4.0):
            rr = O.tree_reward(tree, T, ts["t_lse"], eta)
            assert abs(rr["reward_lse"][r] - sp.logsumexp(eta * vals) / eta) < 1e-12
        assert abs(rew["reward_max"][r] - vals.max()) < 1e-15
        assert abs(rew["reward_mean"][r] - vals.mean()) < 1e-13
        assert rew["n_leaves"][r] == len(vals)


def test_monte_carlo_rollouts_agree_with_nodesum():
    D, T, pool, tree, ts = _case(5, 1, 3, 3, 12, 10, sigma=1.0)
    rew = O.tree_reward(tree, T, ts["t_lse"], 1.0)
    kept, expanded = brute.build_tree(D[0], 3, 3, 10)
    keptset = set(p for p, _ in kept)
    rng = np.random.default_rng(99)
    n = 200000
    lens = np.zeros(n)
    probs = {node: brute.softmax64(T[0, lv, sl]) for node, (lv, sl) in expanded.items()}
    for i in range(n):
        node = ()
        while node in probs:
            tok = int(rng.choice(len(probs[node]), p=probs[node]))
            if node + (tok,) not in keptset:
                break
            node = node + (tok,)
        lens[i] = len(node)
    se = lens.std() / math.sqrt(n)
    assert abs(lens.mean() - rew["reward_nodesum"][0]) < 4 * se + 1e-9


def test_closed_forms_constant_p_and_certain_target():
    # target puts probability p on every kept token: L = p (1 - p^l) / (1 - p)
    R, d, k, V, g = 1, 4, 2, 6, 8
    D, _, pool, tree, _ = _case(8, R, d, k, V, g)
    p = 0.4
    n = int(tree["n_sel"][0])
    T = np.zeros((R, d, k, V))
    t_lse = np.zeros((R, d, k))            # pretend-normalised rows: log prob = log p for every token
    T[:] = math.log(p)
    rew = O.tree_reward(tree, T, t_lse, 1.0)
    for i in range(n):
        l = int(tree["sel_depth"][0, i])
        assert abs(rew["node_cum"][0, i] - p * (1 - p ** l) / (1 - p)) < 1e-13
        assert abs(rew["node_q"][0, i] - p ** l) < 1e-15
    # all-ones target: L_i = l_i, nodesum = number of kept nodes (the upper bound of the reward)
    T[:] = 0.0
    rew = O.tree_reward(tree, T, t_lse, 1.0)
    assert np.allclose(rew["node_cum"][0, :n], tree["sel_depth"][0, :n])
    assert abs(rew["reward_nodesum"][0] - n) < 1e-12


def test_bounds_and_single_sequence():
    D, T, pool, tree, ts = _case(21, 8, 4, 3, 40, 15)
    for eta in (0.5, 1.0, 3.0):
        rew = O.tree_reward(tree, T, ts["t_lse"], eta)
        N = rew["n_leaves"]
        assert (rew["reward_max"] <= rew["reward_lse"] + 1e-12).all()           # App. A Eq. (1)
        assert (rew["reward_lse"] <= rew["reward_max"] + np.log(N) / eta + 1e-12).all()
        assert (rew["reward_nodesum"] <= tree["n_sel"] + 1e-12).all()            # reward <= kept nodes
        assert (rew["reward_nodesum"] <= 4 + 1e-12).all()                        # and <= depth
        assert (rew["reward_mean"] <= rew["reward_max"] + 1e-15).all()
        assert (rew["reward_max"] <= rew["reward_nodesum"] + 1e-12).all()        # one branch is part of the union
    # k = 1: one sequence, so LSE = max = mean = nodesum = L_1
    rng = np.random.default_rng(4)
    D1 = rng.normal(size=(2, 4, 1, 20)); T1 = rng.normal(size=(2, 4, 1, 20))
    st = O.draft_row_stats(D1, 1)
    pool = O.expand_tree(st["top_tok"], st["top_logp32"], 4, 1)
    tree = O.select_topg(pool, 10)
    ts = O.target_row_stats(T1)
    rew = O.tree_reward(tree, T1, ts["t_lse"], 1.0)
    for key in ("reward_max", "reward_mean", "reward_nodesum"):
        np.testing.assert_allclose(rew["reward_lse"], rew[key], rtol=1e-13)


def test_onehot_target_ties_reward_to_greedy_walk():
    """App. A case (b): with a deterministic target every L_i is the common-prefix length
    with the greedy trajectory and max_i L_i is the accepted length."""
    rng = np.random.default_rng(17)
    R, d, k, V, g = 12, 4, 3, 9, 14
    D = rng.normal(0, 1.0, size=(R, d, k, V))
    st = O.draft_row_stats(D, k)
    pool = O.expand_tree(st["top_tok"], st["top_logp32"], d, k)
    tree = O.select_topg(pool, g)
    T = np.full((R, d, k, V), -np.inf)
    # target's certain token: the draft's best token with prob 1/2, else a random token
    for r in range(R):
        for (l, j) in O.used_slots(d, k):
            tok = int(st["top_tok"][r, l, j, 0]) if rng.random() < 0.6 else int(rng.integers(V))
            T[r, l, j, tok] = 0.0
    ts = O.target_row_stats(T)
    rew = O.tree_reward(tree, T, ts["t_lse"], 1.0)
    path = O.accepted_path(tree, ts["t_argmax"], d)
    n = tree["n_sel"]
    for r in range(R):
        cum = rew["node_cum"][r, :n[r]]
        assert np.all(np.abs(cum - np.round(cum)) < 1e-12)
        assert abs(rew["reward_max"][r] - path["path_len"][r]) < 1e-12
        assert abs(rew["reward_nodesum"][r] - path["path_len"][r]) < 1e-12
        kept, expanded = brute.build_tree(D[r], k, d, g)
        walk = brute.greedy_accept([p for p, _ in kept], expanded, T[r], d)
        opaths = brute.oracle_paths(pool, tree, r)
        assert [opaths[i] for i in path["path_node"][r, :path["path_len"][r]]] == [walk[:j + 1] for j in range(len(walk))]
        # path_slot names the row that produced each step
        for t in range(path["path_len"][r]):
            node = walk[:t]
            assert expanded[node] == (t, int(path["path_slot"][r, t]))
        assert (path["path_node"][r, path["path_len"][r]:] == -1).all()
    assert path["path_len"].max() >= 2      # the case really exercises multi-step walks


def test_walk_stops_at_unexpanded_child_and_on_random_targets():
    D, T, pool, tree, ts = _case(33, 10, 4, 3, 8, 20, sigma=2.5)
    path = O.accepted_path(tree, ts["t_argmax"], 4)
    for r in range(10):
        kept, expanded = brute.build_tree(D[r], 3, 4, 20)
        walk = brute.greedy_accept([p for p, _ in kept], expanded, T[r], 4)
        assert path["path_len"][r] == len(walk)


def test_max_l_path_is_the_branch_with_the_largest_expected_length():
    D, T, pool, tree, ts = _case(41, 6, 4, 3, 10, 14)
    rew = O.tree_reward(tree, T, ts["t_lse"], 1.0)
    path = O.max_l_path(tree, rew["node_cum"], 4)
    for r in range(6):
        kept, expanded = brute.build_tree(D[r], 3, 4, 14)
        Ls = brute.sequence_lengths([p for p, _ in kept], expanded, T[r])
        best = max(Ls.values())
        winners = [p for p, L in Ls.items() if L == best]
        assert len(winners) == 1
        opaths = brute.oracle_paths(pool, tree, r)
        l = int(path["path_len"][r])
        assert l == len(winners[0])
        assert [opaths[i] for i in path["path_node"][r, :l]] == [winners[0][:j + 1] for j in range(l)]
        for t in range(l):
            assert expanded[winners[0][:t]] == (t, int(path["path_slot"][r, t]))
        assert (path["path_node"][r, l:] == -1).all() and (path["path_slot"][r, l:] == -1).all()


# ----------------------------------------------------------------- sampled (temperature 1) walk
def _children(tree, r, parent, depth):
    n = int(tree["n_sel"][r])
    return [i for i in range(n) if tree["sel_parent"][r, i] == parent and tree["sel_depth"][r, i] == depth]


def test_sampled_walk_accepts_each_child_with_its_target_probability():
    """Lossless verification: whatever the order of the candidates, the chance that child x is the
    one accepted at a node equals the target probability p(x).  The oracle's acceptance thresholds
    a_1, a_2, ... are found by bisection on the uniform number of each trial (earlier trials forced
    to reject), and prod_{i<j} (1 - a_i) * a_j is compared with scipy's softmax."""
    D, T, pool, tree, ts = _case(7, 1, 3, 3, 12, 10, sigma=1.0)
    d, k = 3, 3

    def thresholds(prefix_u, t, parent):
        kids = _children(tree, 0, parent, t + 1)
        out = []
        for j, kid in enumerate(kids):
            lo, hi = 0.0, 1.0
            for _ in range(60):
                mid = 0.5 * (lo + hi)
                U = np.array(prefix_u, dtype=np.float64).copy()
                U[0, t, :j] = 1.0 - 1e-12          # reject the earlier candidates
                U[0, t, j] = mid
                got = O.sampled_path(tree, T, ts["t_lse"], U, d)
                if got["path_len"][0] > t and got["path_node"][0, t] == kid:
                    lo = mid                       # accepted: the threshold is above mid
                else:
                    hi = mid
            out.append(0.5 * (lo + hi))
        return kids, out

    U0 = np.zeros((1, d, k))
    kids, a = thresholds(U0, 0, -1)
    assert len(kids) >= 2
    p = sp.softmax(T[0, 0, 0])
    keep = 1.0
    for kid, aj in zip(kids, a):
        assert abs(keep * aj - p[tree["sel_tok"][0, kid]]) < 1e-9
        keep *= 1.0 - aj
    # one level down, below the first child (accepted by U = 0 at step 0)
    first = kids[0]
    slot = int(tree["sel_slot"][0, first])
    assert slot >= 0
    kids1, a1 = thresholds(U0, 1, first)
    assert len(kids1) >= 1
    p1 = sp.softmax(T[0, 1, slot])
    keep = 1.0
    for kid, aj in zip(kids1, a1):
        assert abs(keep * aj - p1[tree["sel_tok"][0, kid]]) < 1e-9
        keep *= 1.0 - aj


def test_sampled_walk_mean_length_is_the_nodesum_reward():
    """App. A Eq. (2): the expected number of accepted tokens is the sum over kept nodes of the
    probability that the node is reached; checked by Monte Carlo over the uniform numbers."""
    D, T, pool, tree, ts = _case(5, 1, 3, 3, 12, 10, sigma=1.0)
    rew = O.tree_reward(tree, T, ts["t_lse"], 1.0)
    n = 40000
    rep = {key: np.repeat(val, n, axis=0) for key, val in tree.items() if isinstance(val, np.ndarray) and val.shape[:1] == (1,)}
    Tn = np.broadcast_to(T, (n,) + T.shape[1:])
    lse_n = np.broadcast_to(ts["t_lse"], (n,) + ts["t_lse"].shape[1:])
    U = np.random.default_rng(123).random((n, 3, 3))
    got = O.sampled_path(rep, Tn, lse_n, U, 3)
    lens = got["path_len"].astype(np.float64)
    sigma = lens.std() / math.sqrt(n)
    assert abs(lens.mean() - rew["reward_nodesum"][0]) < 4 * sigma + 1e-12
    # first step: frequency of each depth-1 node against its target probability
    p = sp.softmax(T[0, 0, 0])
    for kid in _children(tree, 0, -1, 1):
        freq = np.mean((got["path_len"] > 0) & (got["path_node"][:, 0] == kid))
        pk = p[tree["sel_tok"][0, kid]]
        assert abs(freq - pk) < 4 * math.sqrt(pk * (1 - pk) / n) + 1e-12


def test_sampled_walk_special_cases():
    D, T, pool, tree, ts = _case(33, 6, 4, 3, 8, 20, sigma=2.5)
    d, k = 4, 3
    # U = 0 accepts the first candidate at every node: the chain of first children in kept order
    got = O.sampled_path(tree, T, ts["t_lse"], np.zeros((6, d, k)), d)
    for r in range(6):
        cur, t = -1, 0
        while t < d:
            kids = _children(tree, r, cur, t + 1)
            if not kids:
                break
            assert got["path_node"][r, t] == kids[0]
            cur = kids[0]
            t += 1
            if tree["sel_slot"][r, cur] < 0:
                break
        assert got["path_len"][r] == t
    # a target that puts (almost) all mass on one token makes the walk the greedy walk for any U
    T2 = T.copy()
    am = ts["t_argmax"]
    for r in range(6):
        for t in range(d):
            for j in range(k):
                T2[r, t, j, am[r, t, j]] += 80.0
    ts2 = O.target_row_stats(T2)
    U = np.random.default_rng(4).random((6, d, k)) * 0.999
    a = O.sampled_path(tree, T2, ts2["t_lse"], U, d)
    b = O.accepted_path(tree, ts2["t_argmax"], d)
    for key in ("path_len", "path_node", "path_slot"):
        assert (a[key] == b[key]).all()
