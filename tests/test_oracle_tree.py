"""Pins for the oracle's tree construction (decoding policy G, Sec. 3.1 (i)-(ii))."""
import json
import math
import os

import numpy as np
import pytest

import brute
from oracle import gto_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def _build(D, k, d, g):
    st = O.draft_row_stats(D, k)
    pool = O.expand_tree(st["top_tok"], st["top_logp32"], d, k, st["top_logp64"], st["top_logit"])
    tree = O.select_topg(pool, g, audit=True)
    return st, pool, tree


def _fig1_logits(fx, probs_key_tree):
    vocab = fx["vocab"]
    k, d = fx["k"], fx["d"]
    V = len(vocab)
    D = np.full((1, d, k, V), -np.inf)

    def fill(l, j, probs):
        for tok, p in probs.items():
            D[0, l, j, vocab.index(tok)] = math.log(p)
    fill(0, 0, probs_key_tree["root"])
    fill(1, 0, probs_key_tree["is"])     # 'is' has the higher root probability -> slot 0
    fill(1, 1, probs_key_tree["has"])
    return D


def _names(fx, paths):
    return ["/".join(fx["vocab"][t] for t in p) for p in paths]


def test_fig1_worked_example_panel_a_and_b():
    fx = json.load(open(os.path.join(HERE, "golden", "fig1_example.json")))
    k, d = fx["k"], fx["d"]
    D = _fig1_logits(fx, fx["draft_probs"])
    # panel (a): top-4 including the root == g = 3 kept nodes
    st, pool, tree = _build(D, k, d, fx["panel_a"]["g"])
    names = _names(fx, brute.oracle_paths(pool, tree, 0))
    assert names == fx["panel_a"]["kept"]
    assert fx["panel_a"]["pruned_greedy"] not in names
    # the confidences the paper prints
    allnames = {}
    for c in range(O.pool_size(d, k)):
        toks, j = [], c
        while j >= 0:
            toks.append(fx["vocab"][pool["cand_tok"][0, j]])
            j = pool["cand_parent"][0, j]
        allnames["/".join(reversed(toks))] = math.exp(pool["cand_score64"][0, c])
    for name, conf in fx["paper_confidences"].items():
        assert abs(allnames[name] - conf) < 1e-12
        assert abs(math.exp(float(pool["cand_score"][0, list(allnames).index(name)])) - conf) < 1e-6
    # panel (b): greedy branch survives (g = 5) but the target accepts a sibling
    st, pool, tree = _build(D, k, d, fx["panel_b"]["g"])
    names = _names(fx, brute.oracle_paths(pool, tree, 0))
    assert names == fx["panel_b"]["kept"]
    T = _fig1_logits(fx, fx["panel_b"]["target_probs"])
    ts = O.target_row_stats(T)
    path = O.accepted_path(tree, ts["t_argmax"], d)
    acc = [names[i] for i in path["path_node"][0, :path["path_len"][0]]]
    assert acc == fx["panel_b"]["accepted"]
    assert acc != fx["panel_b"]["greedy_draft_path"]
    # expected acceptance length of the accepted sequence: 0.7 + 0.7*0.6
    rew = O.tree_reward(tree, T, ts["t_lse"], 1.0)
    i_the = names.index("is/the")
    assert abs(rew["node_cum"][0, i_the] - (0.7 + 0.7 * 0.6)) < 1e-12


@pytest.mark.parametrize("seed,V,k,d,g", [(0, 6, 2, 3, 5), (1, 8, 3, 3, 9), (2, 5, 2, 2, 4),
                                           (3, 7, 3, 2, 50), (4, 8, 2, 3, 3), (5, 8, 3, 3, 20)])
def test_matches_probability_space_brute_force(seed, V, k, d, g):
    rng = np.random.default_rng(seed)
    D = rng.normal(0, 1.5, size=(3, d, k, V))
    st, pool, tree = _build(D, k, d, g)
    for r in range(3):
        kept, expanded = brute.build_tree(D[r], k, d, g)
        assert brute.oracle_paths(pool, tree, r) == [p for p, _ in kept]
        n = int(tree["n_sel"][r])
        np.testing.assert_allclose(np.exp(tree["sel_score"][r, :n].astype(np.float64)),
                                   [c for _, c in kept], rtol=1e-5)
        # slots: the oracle's expanded nodes sit in the same (level, slot)
        paths = brute.oracle_paths(pool, tree, r)
        for i, p in enumerate(paths):
            own = int(tree["sel_slot"][r, i])
            if p in expanded:
                assert expanded[p] == (len(p), own)
            else:
                assert own == -1


def test_structural_invariants_random():
    rng = np.random.default_rng(11)
    R, d, k, V, g = 6, 4, 3, 50, 17
    D = np.round(rng.normal(0, 2, size=(R, d, k, V)) * 4) / 4    # ties on purpose
    st, pool, tree = _build(D, k, d, g)
    C = O.pool_size(d, k)
    assert (tree["n_sel"] == min(g, C)).all()
    for r in range(R):
        n = int(tree["n_sel"][r])
        sc = tree["sel_score"][r, :n]
        assert (np.diff(sc) <= 0).all()                       # kept order is score-descending
        for i in range(n):
            p = int(tree["sel_parent"][r, i])
            assert p < i                                       # parents precede children
            if p >= 0:
                assert tree["sel_depth"][r, i] == tree["sel_depth"][r, p] + 1
                assert sc[i] <= sc[p]                          # confidence never grows along a path
                assert tree["sel_slot"][r, p] == tree["sel_pslot"][r, i]   # parent is expanded, in that slot
            else:
                assert tree["sel_depth"][r, i] == 1 and tree["sel_pslot"][r, i] == 0
            sib = [int(tree["sel_tok"][r, q]) for q in range(n) if tree["sel_parent"][r, q] == p
                   and tree["sel_depth"][r, q] == tree["sel_depth"][r, i]]
            assert len(set(sib)) == len(sib)                   # distinct tokens among siblings
        for l in range(1, d):
            exp_nodes = pool["slot_cand"][r, l]
            assert len(set(exp_nodes.tolist())) == k and (exp_nodes >= 0).all()
            assert (pool["cand_depth"][r, exp_nodes] == l).all()
        assert (pool["slot_cand"][r, 0] == -1).all()


def test_k1_is_greedy_chain():
    rng = np.random.default_rng(3)
    d, V = 5, 30
    D = rng.normal(size=(2, d, 1, V))
    st, pool, tree = _build(D, 1, d, 60)
    for r in range(2):
        assert tree["n_sel"][r] == d
        assert tree["sel_tok"][r, :d].tolist() == [int(np.argmax(D[r, l, 0])) for l in range(d)]
        assert tree["sel_parent"][r, :d].tolist() == [-1, 0, 1, 2, 3]
        assert tree["sel_leaf"][r, :d].tolist() == [0, 0, 0, 0, 1]


def test_g_at_least_C_keeps_everything_and_onehot_rows_tie_break_by_index():
    d, k, V = 3, 2, 9
    C = O.pool_size(d, k)
    D = np.full((1, d, k, V), -np.inf)
    D[..., 4] = 0.0                                           # one-hot rows: logp = 0 for token 4
    st, pool, tree = _build(D, k, d, C + 5)
    assert tree["n_sel"][0] == C
    # scores: rank-0 children have score 0, rank-1 children -inf; order is by pool index inside ties
    zero = [c for c in range(C) if pool["cand_score"][0, c] == 0.0]
    assert tree["sel_cand"][0, :len(zero)].tolist() == zero
    rest = [c for c in range(C) if c not in zero]
    assert tree["sel_cand"][0, len(zero):C].tolist() == rest
    assert (tree["sel_cand"][0, C:] == -1).all()


def test_margin_audit_flags_near_ties_only():
    d, k, V = 2, 2, 6
    D = np.full((1, d, k, V), -20.0)
    D[0, 0, 0, 0], D[0, 0, 0, 1] = 2.0, 1.0
    D[0, 1, 0, 2], D[0, 1, 0, 3] = 3.0, 1.0
    D[0, 1, 1, 4], D[0, 1, 1, 5] = 3.0, 0.5
    _, pool, tree = _build(D, k, d, 3)
    assert tree["min_margin"][0] > 1e3 and pool["min_margin"][0] == np.inf   # clear by a wide margin
    # move the third-ranked candidate to within 1e-9 of the second (they are not parent and child)
    order = sorted(range(6), key=lambda c: (-pool["cand_score64"][0, c], c))
    hi, lo = order[1], order[2]
    assert pool["cand_parent"][0, lo] != hi and pool["cand_parent"][0, hi] != lo
    gap = pool["cand_score64"][0, hi] - pool["cand_score64"][0, lo]
    assert gap > 0
    pool["cand_score64"][0, lo] += gap - 1e-9
    assert O.select_topg(pool, 3, audit=True)["min_margin"][0] < 1.0
    # a gap of about one fp32 ulp of the scores is still flagged, a gap of 1e-4 is not
    pool["cand_score64"][0, lo] -= 1e-7
    assert O.select_topg(pool, 3, audit=True)["min_margin"][0] < 1.0
    pool["cand_score64"][0, lo] -= 1e-4
    assert O.select_topg(pool, 3, audit=True)["min_margin"][0] > 1.0
    # a child within rounding of its own parent is never a near tie: the parent always ranks first
    child = [c for c in range(6) if pool["cand_parent"][0, c] == order[0]][0]
    pool["cand_score64"][0, child] = pool["cand_score64"][0, order[0]] - 1e-12
    assert O.select_topg(pool, 3, audit=True)["min_margin"][0] > 1.0
    # exact ties that every arithmetic resolves alike (parent/child at logp 0, -inf against -inf)
    D3 = np.full((1, d, k, V), -np.inf)
    D3[0, 0, 0, 1], D3[0, 1, 0, 2], D3[0, 1, 1, 3] = 0.0, 0.0, 0.0
    _, pool3, tree3 = _build(D3, k, d, 5)          # kept: the chain 1 -> 2, then -inf candidates by index
    assert tree3["sel_cand"][0].tolist() == [0, 2, 1, 3, 4] and tree3["min_margin"][0] == np.inf


def _two_candidate_pool(lp_a, lp_b, logit_err):
    """d = 1, k = 2: the root's two children are the whole pool; their scores are their log-probabilities."""
    top_tok = np.array([[[[0, 1], [0, 0]]]], dtype=np.int32)                    # [R=1, d=1, k=2, k=2]
    lp64 = np.array([[[[lp_a, lp_b], [0.0, 0.0]]]])
    logit = np.array([[[[1.0, 0.5], [0.0, 0.0]]]])                              # distinct logits: not an exact tie
    return O.expand_tree(top_tok, lp64.astype(np.float32), 1, 2, lp64, logit, logit_err)


def test_logit_error_budget_straddle():
    """The audit's budget with an absolute logit error E (fused LM-head workload): each log-probability may be
    off by 2 E (its logit by E, its row's log-sum-exp by E), on top of the fp32 terms.  Two candidates whose
    gap is just above 2 x (budget_a + budget_b) are clear, just below it they are a near tie; without E the
    same gap is clear by a wide margin."""
    E = 1e-3
    lp_a = -0.5
    fp32_terms = lambda lp: float(np.spacing(np.float32(abs(lp)))) + 2.0 ** -23
    for factor, clear in ((1.02, True), (0.98, False)):
        # solve gap = factor * 2 * (budget_a + budget_b); the budget of b depends (weakly) on lp_b through its ulp
        gap = factor * 2.0 * (fp32_terms(lp_a) + fp32_terms(lp_a - 8.0 * E) + 4.0 * E)
        pool = _two_candidate_pool(lp_a, lp_a - gap, E)
        tree = O.select_topg(pool, 1, audit=True)
        assert (tree["min_margin"][0] >= 1.0) == clear, (factor, tree["min_margin"][0])
        assert abs(tree["min_margin"][0] - factor) < 0.01
        # the budget itself: fp32 terms + 2 E per candidate
        assert abs(pool["cand_err"][0, 0] - (fp32_terms(lp_a) + 2 * E)) < 1e-12
        wide = O.select_topg(_two_candidate_pool(lp_a, lp_a - gap, 0.0), 1, audit=True)
        assert wide["min_margin"][0] > 1e3


def test_logit_error_budget_is_sound_against_perturbed_logits():
    """What the budget is for, checked by brute force: if the audit calls a root clear (ratio >= 1) under a
    logit error E, then no perturbation of the log-probabilities by up to 2 E each (all 2^C corners, fp32
    scores recomputed) changes the kept set or its order; and a gap smaller than the two candidates' combined
    2 E allowances is always flagged."""
    rng = np.random.default_rng(11)
    E = 2e-3
    k, d = 4, 1
    n_clear = n_flagged = 0
    for it in range(300):
        lp = -np.sort(rng.uniform(0.05, 0.12, size=k)).astype(np.float64) - np.arange(k) * rng.choice([0.0, 0.004, 0.03])
        top_tok = np.zeros((1, d, k, k), dtype=np.int32)
        top_tok[0, 0, 0] = np.arange(k)
        lp64 = np.zeros((1, d, k, k))
        lp64[0, 0, 0] = lp
        logit = np.zeros((1, d, k, k))
        logit[0, 0, 0] = 5.0 - np.arange(k)
        pool = O.expand_tree(top_tok, lp64.astype(np.float32), d, k, lp64, logit, E)
        tree = O.select_topg(pool, 2, audit=True)
        base = tree["sel_cand"][0].tolist()
        flips = False
        for corner in range(1 << k):
            delta = np.array([(2 * E if (corner >> i) & 1 else -2 * E) for i in range(k)])
            pert = lp64.copy()
            pert[0, 0, 0] = lp + delta
            p2 = O.expand_tree(top_tok, pert.astype(np.float32), d, k)
            if O.select_topg(p2, 2)["sel_cand"][0].tolist() != base:
                flips = True
                break
        gaps = np.abs(np.diff(lp[:3]))                    # the audited neighbours: ranks (0,1) and (1,2)
        if tree["min_margin"][0] >= 1.0:
            n_clear += 1
            assert not flips, (it, lp, tree["min_margin"][0])
        if gaps.min() < 4 * E:                            # inside the two candidates' allowances: must be flagged
            n_flagged += 1
            assert tree["min_margin"][0] < 1.0, (it, lp)
    assert n_clear > 20 and n_flagged > 20
