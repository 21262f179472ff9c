"""Plain CPU oracle for the Group Tree Optimization (GTO) hot path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
what the HIP library computes.  Nothing in the product path may import it; only
tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code
with the HIP kernels, their headers or their Python binding, and imports neither.

Everything is written per root with plain loops and numpy library primitives
(sort, exp, log).  Floating point is fp64, with one deliberate exception: the
ranking key of a tree node (its cumulative draft log-probability) is an fp32
value, because the method's ranking decisions are defined on fp32 scores; the
fp64 twin of every score is carried next to it so that a test can tell a clear
decision from a near tie.

Passages followed (paper: "Bridging Draft Policy Misalignment: Group Tree
Optimization for Speculative Decoding"):
  * Sec. 3.1 "Draft Tree Reward": decoding policy G, stage (i) layer-wise
    expansion and stage (ii) global re-ranking; Eq. 2-5 (sequence set, expected
    acceptance length of a sequence, prefix probability, smooth-max reward).
  * Fig. 1 caption: edge number = draft token probability, number in parentheses
    = path confidence = product of the edge probabilities from the root (1.0).
  * Sec. 4 ablation "Aggregation Operator": the Max and Mean aggregates.
  * App. A Eq. (2) and Lemma 1: expected decoding length as a sum over disjoint
    prefix events (= sum over distinct tree nodes of the accepted-prefix
    probability); T=0 case: acceptance follows the greedy target trajectory.
  * Sec. 3.2 "Tree Reward Optimization": Eq. 6-7 grouping, Eq. 9 debiased reward,
    Eq. 10 group standardisation, Eq. 11 geometric-mean likelihood ratio on the
    longest accepted sequence, Eq. 12 clipped surrogate; Algorithm 1.
  * Eq. 13 and App. B.2: token-level cross-entropy from the target to the draft distribution.
  * App. B.1/B.3: k = 10, g = 60, depth 7, eta = 1, m = 8.
  * Sec. 4 "Metrics": evaluation at temperatures 0 and 1; the temperature-1 reading of the longest
    accepted sequence (sampled_path) is the lossless acceptance rule for deterministically chosen
    candidates, whose expectation is the node-sum of App. A Eq. (2).
  * Fused LM-head variant: logits = hidden . W^T (fused_logits); the hidden-state gradient is the
    chain rule through that product (ppo_surrogate_bwd_dh).

Readings where the paper is silent (each is repeated next to the code it affects):
  tie-breaks are lowest token id / lowest pool index; g counts kept nodes (root
  excluded) among all generated candidates; softmax is over the full vocabulary at
  temperature 1; std is the population std; the l = 0 case uses max(l, 1);
  advantages are constants for the gradient; a ratio exactly on the clip boundary
  counts as unclipped.

Pins (see tests/test_oracle_*.py): every function here is pinned; none is
"parity unpinned".

Layouts (R roots, d levels, k branching, V vocabulary, C = k + (d-1) k^2):
  logits            [R, d, k, V]   slot (l, j) = distribution at the j-th expanded
                                   node of level l; level 0 uses slot (0, 0) only.
  pool index c      c = r                          for the root's r-th child
                    c = k + (l-1) k^2 + j k + r    for the r-th child of slot (l, j)
"""
from __future__ import annotations

import math

import numpy as np

NEG_INF = float("-inf")


def used_slots(d: int, k: int):
    """Slots whose rows are read: (0,0) and (l, j) for 1 <= l < d, 0 <= j < k."""
    out = [(0, 0)]
    for l in range(1, d):
        for j in range(k):
            out.append((l, j))
    return out


def pool_size(d: int, k: int) -> int:
    return k + (d - 1) * k * k


# --------------------------------------------------------------------------- rows
def fused_logits(H: np.ndarray, W_vh: np.ndarray) -> np.ndarray:
    """Logits of the fused LM-head workload: logits[r, l, j, v] = sum_h H[r, l, j, h] * W_vh[v, h], in
    fp64 (inputs are bf16 values, so every product is exact and only the fp64 sum rounds).  Rows of
    padding slots are left at zero; they are never read."""
    R, d, k, Hd = H.shape
    V = W_vh.shape[0]
    W64 = W_vh.astype(np.float64, copy=False)
    slots = used_slots(d, k)
    out = np.zeros((R, d, k, V))
    for r in range(R):
        rows = np.stack([H[r, l, j] for (l, j) in slots]).astype(np.float64)      # [rho, Hd]
        prod = rows @ W64.T                                                       # one matmul per root
        for i, (l, j) in enumerate(slots):
            out[r, l, j] = prod[i]
    return out


def fp32_accumulation_error(hidden: int, max_abs_logit: float) -> float:
    """Absolute error to grant a logit that the other side accumulates in fp32 on the matrix cores, where this
    oracle accumulates in fp64 (the `logit_err` of row_margins and expand_tree).  The fp32 accumulator is
    rounded once per step of 16 products, i.e. hidden / 16 times; each rounding is uniform within half an ulp
    of the running sum, which stays below the largest |logit|, so one rounding has a standard deviation of at
    most ulp32(max |logit|) / sqrt(12), and their sum sqrt(hidden / 16) times that.  The bound is six such
    standard deviations: a full-size comparison checks ~1e5 logits against it, and a bound that one of them
    may exceed by chance would be useless (the worst case, hidden / 16 half-ulps, is never approached)."""
    return 6.0 * _ulp32(max_abs_logit) * math.sqrt(max(hidden / 16.0, 1.0) / 12.0)


def row_margins(logits: np.ndarray, k: int, logit_err: float) -> np.ndarray:
    """Near-tie audit of the per-row top-k when the logits themselves carry an error of up to
    `logit_err` (fp32 accumulation on the other side): per root, the smallest gap between
    neighbours among the k+1 largest logits of any used row, divided by 2 * logit_err.  Below 1
    the order of that row's top-k (or its cut) may legitimately differ."""
    R, d, kk, V = logits.shape
    out = np.full((R,), np.inf)
    for r in range(R):
        for (l, j) in used_slots(d, kk):
            top = np.sort(logits[r, l, j])[::-1][: k + 1]
            gaps = top[:-1] - top[1:]
            if len(gaps):
                out[r] = min(out[r], float(gaps.min()) / (2.0 * logit_err))
    return out


def _row_lse(x64: np.ndarray):
    m = float(np.max(x64))
    s = float(np.sum(np.exp(x64 - m)))
    return m, m + math.log(s)


def draft_row_stats(D: np.ndarray, k: int):
    """Per used slot: max, log-sum-exp and the k most probable tokens.

    Fig. 1 caption / Sec. 3.1 (i): every expanded node proposes its top-k tokens
    with their draft probabilities.  The softmax is taken over the whole
    vocabulary (no renormalisation over the k kept tokens).  Order: logit
    descending, token id ascending among equal logits (a full stable sort of the
    negated row is the definition used).

    Returns dict with row_max, row_lse (fp64), top_tok (int32), top_logit (fp64),
    top_logp64 (fp64) and top_logp32 = fp32(top_logp64), the ranking increment.
    """
    R, d, kk, V = D.shape
    assert kk == k and V >= k
    row_max = np.full((R, d, k), np.nan)
    row_lse = np.full((R, d, k), np.nan)
    top_tok = np.full((R, d, k, k), -1, dtype=np.int32)
    top_logit = np.full((R, d, k, k), np.nan)
    top_logp64 = np.full((R, d, k, k), np.nan)
    for r in range(R):
        for (l, j) in used_slots(d, k):
            x = D[r, l, j].astype(np.float64)
            m, lse = _row_lse(x)
            order = np.argsort(-x, kind="stable")[:k]
            row_max[r, l, j] = m
            row_lse[r, l, j] = lse
            top_tok[r, l, j] = order
            top_logit[r, l, j] = x[order]
            top_logp64[r, l, j] = x[order] - lse
    with np.errstate(invalid="ignore"):
        top_logp32 = top_logp64.astype(np.float32)
    return dict(row_max=row_max, row_lse=row_lse, top_tok=top_tok, top_logit=top_logit,
                top_logp64=top_logp64, top_logp32=top_logp32)


def target_row_stats(T: np.ndarray):
    """Per used slot of the target logits: max, argmax (lowest id) and lse.

    Needed by Eq. 3-4 (target probability of a drafted token) and by the greedy
    (T=0) verification walk of App. A case (b).
    """
    R, d, k, V = T.shape
    t_max = np.full((R, d, k), np.nan)
    t_lse = np.full((R, d, k), np.nan)
    t_argmax = np.full((R, d, k), -1, dtype=np.int32)
    for r in range(R):
        for (l, j) in used_slots(d, k):
            x = T[r, l, j].astype(np.float64)
            m, lse = _row_lse(x)
            t_max[r, l, j] = m
            t_lse[r, l, j] = lse
            t_argmax[r, l, j] = int(np.argmax(x))  # first occurrence = lowest id
    return dict(t_max=t_max, t_lse=t_lse, t_argmax=t_argmax)


# ---------------------------------------------------------------------- expansion
def _ranked(indices, score32):
    """Indices sorted by (fp32 score descending, index ascending)."""
    return sorted(indices, key=lambda c: (-float(score32[c]), c))


AUDIT_SAFETY = 2.0
SUM_REL_ERR = 2.0 ** -23      # relative accuracy granted to an fp32 sum of exponentials


def _ulp32(x) -> float:
    x = abs(float(x))
    return float(np.spacing(np.float32(x))) if math.isfinite(x) else 0.0


def _gap_audit(order, upto, score64, parent, logit, err, margin):
    """Near-tie audit of one ranking decision.  For each pair of neighbours among the first
    `upto`+1 ranked entries: fp64 score gap divided by AUDIT_SAFETY times the sum of the two
    candidates' fp32 error budgets (`err`, see expand_tree).  A ratio below 1 means that an
    implementation whose row statistics differ from this one by fp32 rounding may rank the pair
    the other way; both orders are then correct.  Skipped, because every arithmetic resolves them
    alike: two children of one parent with the same logit and two scores of -inf (index order), and
    a node next to its own parent (a log-probability is <= 0 and the parent's index is lower)."""
    n = min(upto + 1, len(order))
    for a, b in zip(order[: n - 1], order[1:n]):
        if parent[a] == parent[b] and logit is not None and logit[a] == logit[b]:
            continue
        if parent[b] == a or parent[a] == b:
            continue
        ga, gb = score64[a], score64[b]
        if ga == gb and ga == NEG_INF:
            continue
        gap = 0.0 if ga == gb else abs(ga - gb)
        budget = AUDIT_SAFETY * (err[a] + err[b])
        ratio = gap / budget if budget > 0 else (np.inf if gap > 0 else 0.0)
        if ratio < margin[0]:
            margin[0] = ratio
    return margin


def expand_tree(top_tok, top_logp32, d: int, k: int, top_logp64=None, top_logit=None, logit_err: float = 0.0):
    """Stage (i) of the decoding policy G: layer-wise expansion.

    Level 0: the root (path confidence 1.0, i.e. score 0) proposes k children,
    all of which become the expanded nodes (slots) of level 1 in rank order.
    Level l >= 1: each of the k slots proposes k children; a child's global
    acceptance score is its parent's score plus its own draft log-probability
    (Fig. 1 caption: confidences multiply).  While l < d-1, the k best of those
    k^2 children (score descending, pool index ascending) become slots
    (l+1, 0..k-1) in that order; the others stay unexpanded candidates.

    The score is an fp32 value: score = fp32(score_parent + logp32).  If
    `top_logp64` is given the fp64 twin is accumulated too, together with an error
    budget per candidate, err = err(parent) + ulp32(logp) + 2^-23 + ulp32(score)/2
    (an implementation's fp32 log-probability may be one ulp away from this one's,
    its sum of exponentials is only accurate to fp32 relative precision, and each
    fp32 add rounds by half an ulp); `min_margin[r]` is then the smallest
    gap-to-budget ratio (see _gap_audit) over the ranking decisions of root r:
    >= 1 means every decision of that root is clear of fp32 rounding.  `logit_err` adds, per
    level, twice an absolute error of the logits themselves (fused LM-head workload, where the
    other side accumulates the logits in fp32): once for the logit, once for the row's lse.

    Returns dict: cand_tok, cand_parent (pool index or -1), cand_depth (1..d),
    cand_pslot (slot j of the parent within its level), cand_slot (slot the node
    itself occupies if expanded, else -1) [R, C] int32; cand_score [R, C] fp32;
    cand_score64 [R, C]; slot_cand [R, d, k] int32 (pool index expanded in each
    slot; (0,0) is the root = -1; unused level-0 slots -1); min_margin [R].
    """
    R = top_tok.shape[0]
    C = pool_size(d, k)
    kk = k * k
    cand_tok = np.full((R, C), -1, dtype=np.int32)
    cand_parent = np.full((R, C), -1, dtype=np.int32)
    cand_depth = np.zeros((R, C), dtype=np.int32)
    cand_pslot = np.zeros((R, C), dtype=np.int32)
    cand_slot = np.full((R, C), -1, dtype=np.int32)
    cand_score = np.zeros((R, C), dtype=np.float32)
    cand_score64 = np.zeros((R, C), dtype=np.float64)
    cand_logit = np.zeros((R, C), dtype=np.float64)
    cand_err = np.zeros((R, C), dtype=np.float64)
    slot_cand = np.full((R, d, k), -1, dtype=np.int32)
    min_margin = np.full((R,), np.inf)
    lp64 = top_logp64 if top_logp64 is not None else top_logp32.astype(np.float64)
    for r in range(R):
        margin = [np.inf]
        # level 0: children of the root
        for rank in range(k):
            c = rank
            cand_tok[r, c] = top_tok[r, 0, 0, rank]
            cand_parent[r, c] = -1
            cand_depth[r, c] = 1
            cand_pslot[r, c] = 0
            cand_score[r, c] = np.float32(0.0) + np.float32(top_logp32[r, 0, 0, rank])
            cand_score64[r, c] = lp64[r, 0, 0, rank]
            cand_err[r, c] = _ulp32(top_logp32[r, 0, 0, rank]) + SUM_REL_ERR + 2.0 * logit_err
            if top_logit is not None:
                cand_logit[r, c] = top_logit[r, 0, 0, rank]
        if d > 1:
            for rank in range(k):
                slot_cand[r, 1, rank] = rank
                cand_slot[r, rank] = rank
        for l in range(1, d):
            base = k + (l - 1) * kk
            for j in range(k):
                p = int(slot_cand[r, l, j])
                for rank in range(k):
                    c = base + j * k + rank
                    cand_tok[r, c] = top_tok[r, l, j, rank]
                    cand_parent[r, c] = p
                    cand_depth[r, c] = l + 1
                    cand_pslot[r, c] = j
                    cand_score[r, c] = np.float32(cand_score[r, p]) + np.float32(top_logp32[r, l, j, rank])
                    cand_score64[r, c] = cand_score64[r, p] + lp64[r, l, j, rank]
                    cand_err[r, c] = cand_err[r, p] + _ulp32(top_logp32[r, l, j, rank]) + SUM_REL_ERR + 2.0 * logit_err \
                        + 0.5 * _ulp32(cand_score[r, c])
                    if top_logit is not None:
                        cand_logit[r, c] = top_logit[r, l, j, rank]
            if l < d - 1:
                order = _ranked(range(base, base + kk), cand_score[r])
                for i in range(k):
                    slot_cand[r, l + 1, i] = order[i]
                    cand_slot[r, order[i]] = i
                if top_logp64 is not None:
                    _gap_audit(order, k, cand_score64[r], cand_parent[r],
                               cand_logit[r] if top_logit is not None else None, cand_err[r], margin)
        min_margin[r] = margin[0]
    return dict(cand_tok=cand_tok, cand_parent=cand_parent, cand_depth=cand_depth,
                cand_pslot=cand_pslot, cand_slot=cand_slot, cand_score=cand_score,
                cand_score64=cand_score64, cand_logit=cand_logit, cand_err=cand_err, slot_cand=slot_cand,
                min_margin=min_margin)


def select_topg(pool, g: int, audit: bool = False):
    """Stage (ii) of G: global re-ranking, keep the g best, prune the rest.

    All C generated candidates of all depths compete on the global acceptance
    score (fp32, descending; pool index ascending among equals); the first
    min(g, C) are kept, in that order.  Because a log-probability is <= 0 and fp32
    addition is monotone, a child never outranks its parent, so the kept set is
    closed under taking parents and every kept node's parent precedes it.

    Returns dict (all [R, g], unused tail = -1 / 0): sel_cand (pool index),
    sel_tok, sel_parent (position of the parent in the kept list, -1 for depth-1
    nodes), sel_depth, sel_pslot, sel_slot, sel_leaf (1 if no kept child),
    sel_score fp32; n_sel [R]; slot_need [R, d, k] (1 for every slot whose node has a
    kept child, i.e. whose target row the reward reads); min_margin [R] (near-tie audit over the kept
    order and the cut, only if audit=True; see _gap_audit).
    """
    cand_score = pool["cand_score"]
    R, C = cand_score.shape
    n_keep = min(g, C)
    sel = {name: np.full((R, g), -1, dtype=np.int32)
           for name in ("sel_cand", "sel_tok", "sel_parent", "sel_depth", "sel_pslot", "sel_slot")}
    sel["sel_depth"][:] = 0
    sel["sel_pslot"][:] = 0
    sel_leaf = np.zeros((R, g), dtype=np.int32)
    sel_score = np.zeros((R, g), dtype=np.float32)
    n_sel = np.full((R,), n_keep, dtype=np.int32)
    d_levels, k_slots = pool["slot_cand"].shape[1:]
    slot_need = np.zeros((R, d_levels, k_slots), dtype=np.int32)
    min_margin = np.full((R,), np.inf)
    for r in range(R):
        order = _ranked(range(C), cand_score[r])
        kept = order[:n_keep]
        pos = {c: i for i, c in enumerate(kept)}
        has_child = [False] * n_keep
        for i, c in enumerate(kept):
            p = int(pool["cand_parent"][r, c])
            if p >= 0:
                if p not in pos or pos[p] >= i:
                    raise AssertionError("kept set is not closed under parents")
                has_child[pos[p]] = True
            sel["sel_cand"][r, i] = c
            sel["sel_tok"][r, i] = pool["cand_tok"][r, c]
            sel["sel_parent"][r, i] = pos[p] if p >= 0 else -1
            sel["sel_depth"][r, i] = pool["cand_depth"][r, c]
            sel["sel_pslot"][r, i] = pool["cand_pslot"][r, c]
            sel["sel_slot"][r, i] = pool["cand_slot"][r, c]
            sel_score[r, i] = cand_score[r, c]
            # the target row at the parent's slot is what Eq. 4 reads for this node
            slot_need[r, int(pool["cand_depth"][r, c]) - 1, int(pool["cand_pslot"][r, c])] = 1
        for i in range(n_keep):
            sel_leaf[r, i] = 0 if has_child[i] else 1
        if audit:
            margin = [np.inf]
            _gap_audit(order, n_keep, pool["cand_score64"][r], pool["cand_parent"][r],
                       pool.get("cand_logit", [None] * R)[r], pool["cand_err"][r], margin)
            min_margin[r] = margin[0]
    out = dict(sel)
    out.update(sel_leaf=sel_leaf, sel_score=sel_score, n_sel=n_sel, slot_need=slot_need, min_margin=min_margin)
    return out


# ------------------------------------------------------------------------- reward
def tree_reward(tree, T: np.ndarray, t_lse: np.ndarray, eta: float = 1.0):
    """Draft Tree Reward, Eq. 2-5, plus the ablation aggregates and App. A Eq. (2).

    For a kept node n at depth j on a root-to-leaf sequence, the target
    probability that the first j tokens are all accepted is the product of the
    target's conditional token probabilities along the path (Eq. 4); the target
    distribution for a node's token is the softmax of the target logits at the
    node's parent (slot `sel_pslot` of level depth-1).  The expected acceptance
    length of a sequence is the sum of these prefix probabilities over its nodes
    (Eq. 3).  Sequences are the root-to-leaf paths of the kept tree, a leaf being
    a kept node with no kept child (Eq. 2).

    Outputs: node_q [R, g] prefix probability of each kept node, node_cum [R, g]
    running sum along the path (= L of the sequence at a leaf), and per root
      lse     = (1/eta) log sum_i exp(eta L_i)            (Eq. 5, no 1/N inside)
      max     = max_i L_i,   mean = (1/N) sum_i L_i        (ablation variants)
      nodesum = sum over kept nodes of node_q              (App. A Eq. (2): the
                prefix events of distinct nodes at one depth are disjoint)
    """
    R, g = tree["sel_tok"].shape
    node_q = np.zeros((R, g))
    node_cum = np.zeros((R, g))
    agg = dict(lse=np.zeros(R), max=np.zeros(R), mean=np.zeros(R), nodesum=np.zeros(R))
    n_leaves = np.zeros(R, dtype=np.int32)
    for r in range(R):
        n = int(tree["n_sel"][r])
        logq = np.zeros(n)
        Ls = []
        for i in range(n):
            p = int(tree["sel_parent"][r, i])
            lvl = int(tree["sel_depth"][r, i]) - 1
            j = int(tree["sel_pslot"][r, i])
            tok = int(tree["sel_tok"][r, i])
            logt = float(T[r, lvl, j, tok]) - float(t_lse[r, lvl, j])
            logq[i] = (logq[p] if p >= 0 else 0.0) + logt
            q = math.exp(logq[i])
            node_q[r, i] = q
            node_cum[r, i] = (node_cum[r, p] if p >= 0 else 0.0) + q
        for i in range(n):
            if tree["sel_leaf"][r, i]:
                Ls.append(node_cum[r, i])
        Ls = np.asarray(Ls)
        n_leaves[r] = len(Ls)
        if len(Ls):
            mx = float(Ls.max())
            agg["lse"][r] = mx + math.log(float(np.sum(np.exp(eta * (Ls - mx))))) / eta
            agg["max"][r] = mx
            agg["mean"][r] = float(Ls.mean())
        agg["nodesum"][r] = float(node_q[r, :n].sum())
    return dict(node_q=node_q, node_cum=node_cum, reward_lse=agg["lse"], reward_max=agg["max"],
                reward_mean=agg["mean"], reward_nodesum=agg["nodesum"], n_leaves=n_leaves)


def accepted_path(tree, t_argmax: np.ndarray, d: int):
    """Longest accepted sequence under the target (Sec. 3.2, Algorithm 1), read as
    greedy (T=0) verification, App. A case (b): starting at the root, accept the
    kept child whose token equals the target's argmax at the current node, and
    continue from that child while it is itself an expanded node (so that the
    target distribution after it is known) and depth remains.

    Returns path_len [R] (0..d), path_node [R, d] (positions in the kept list, -1
    beyond the length) and path_slot [R, d] (slot, within level t, of the node
    whose distribution produced step t; -1 beyond the length).
    """
    R, g = tree["sel_tok"].shape
    path_len = np.zeros(R, dtype=np.int32)
    path_node = np.full((R, d), -1, dtype=np.int32)
    path_slot = np.full((R, d), -1, dtype=np.int32)
    for r in range(R):
        n = int(tree["n_sel"][r])
        cur, slot = -1, 0
        for t in range(d):
            want = int(t_argmax[r, t, slot])
            nxt = -1
            for i in range(n):
                if int(tree["sel_parent"][r, i]) == cur and int(tree["sel_depth"][r, i]) == t + 1 \
                        and int(tree["sel_tok"][r, i]) == want:
                    nxt = i
                    break
            if nxt < 0:
                break
            path_node[r, t] = nxt
            path_slot[r, t] = slot
            path_len[r] = t + 1
            own = int(tree["sel_slot"][r, nxt])
            if own < 0:
                break
            cur, slot = nxt, own
    return dict(path_len=path_len, path_node=path_node, path_slot=path_slot)


def max_l_path(tree, node_cum: np.ndarray, d: int):
    """Alternative reading of the "longest accepted sequence" (Sec. 3.2): the root-to-leaf sequence
    of the kept tree whose expected acceptance length L_i (Eq. 3) is largest, the first such leaf
    in kept order among equals.  Same outputs as accepted_path; the length is the leaf's depth."""
    R, g = tree["sel_tok"].shape
    path_len = np.zeros(R, dtype=np.int32)
    path_node = np.full((R, d), -1, dtype=np.int32)
    path_slot = np.full((R, d), -1, dtype=np.int32)
    for r in range(R):
        n = int(tree["n_sel"][r])
        best, bl = -1, -1.0
        for i in range(n):
            if tree["sel_leaf"][r, i] and node_cum[r, i] > bl:
                best, bl = i, node_cum[r, i]
        chain = []
        p = best
        while p >= 0:
            chain.append(p)
            p = int(tree["sel_parent"][r, p])
        chain.reverse()
        path_len[r] = len(chain)
        for t, node in enumerate(chain):
            path_node[r, t] = node
            path_slot[r, t] = tree["sel_pslot"][r, node]
    return dict(path_len=path_len, path_node=path_node, path_slot=path_slot)


def sampled_path(tree, T: np.ndarray, t_lse: np.ndarray, U: np.ndarray, d: int):
    """Third reading of the "longest accepted sequence" (Sec. 3.2; Sec. 4 evaluates at temperature
    1 as well): the sequence that lossless verification at temperature 1 accepts.  The tree's
    children were chosen deterministically (top-k), so each candidate is a point proposal: at the
    current node, with target distribution p = softmax(target row), the kept children are tried in
    kept order; child x is accepted with probability p(x) / (1 - mass of the children already
    rejected at this node), i.e. p renormalised without the rejected tokens.  Acceptance moves to
    that child, and the walk goes on while the child is itself expanded and depth remains; if
    every child is rejected the walk ends.  The chance that child x is the one accepted is then
    exactly p(x), which is what keeps the procedure lossless and makes the expected length equal
    the node-sum reward of App. A Eq. (2).

    U [R, d, k] holds the uniform numbers in [0, 1): U[r, t, j] decides the j-th child tried at
    step t (a child is accepted iff U < its acceptance probability).  Outputs as accepted_path,
    plus `margin` [R]: the smallest |U - acceptance probability| over the decisions taken (a
    comparison in lower precision can only differ where this is tiny)."""
    R, g = tree["sel_tok"].shape
    path_len = np.zeros(R, dtype=np.int32)
    path_node = np.full((R, d), -1, dtype=np.int32)
    path_slot = np.full((R, d), -1, dtype=np.int32)
    margin = np.full(R, np.inf)
    for r in range(R):
        n = int(tree["n_sel"][r])
        cur, slot = -1, 0
        for t in range(d):
            rest = 1.0                       # target mass not yet rejected at this node
            j = 0
            nxt = -1
            for i in range(n):
                if int(tree["sel_parent"][r, i]) != cur or int(tree["sel_depth"][r, i]) != t + 1:
                    continue
                tok = int(tree["sel_tok"][r, i])
                p_tok = math.exp(float(T[r, t, slot, tok]) - float(t_lse[r, t, slot]))
                acc = p_tok / rest if rest > 0.0 else 1.0
                u = float(U[r, t, j])
                margin[r] = min(margin[r], abs(u - acc))
                if u < acc:
                    nxt = i
                    break
                rest -= p_tok
                j += 1
            if nxt < 0:
                break
            path_node[r, t] = nxt
            path_slot[r, t] = slot
            path_len[r] = t + 1
            own = int(tree["sel_slot"][r, nxt])
            if own < 0:
                break
            cur, slot = nxt, own
    return dict(path_len=path_len, path_node=path_node, path_slot=path_slot, margin=margin)


# ---------------------------------------------------------------------- advantage
def group_advantage(r_cur, r_ref, m: int, delta: float = 1e-6):
    """Eq. 9-10: debias against the reference tree, then standardise inside each
    group of m consecutive roots with the population std (ddof = 0) plus delta.
    r_ref = None gives the "without debiasing" ablation variant."""
    r_cur = np.asarray(r_cur, dtype=np.float64)
    Rdeb = r_cur - (np.asarray(r_ref, dtype=np.float64) if r_ref is not None else 0.0)
    R = Rdeb.shape[0]
    assert R % m == 0
    adv = np.zeros(R)
    for g0 in range(0, R, m):
        grp = Rdeb[g0:g0 + m]
        mean = grp.sum() / m
        std = math.sqrt(((grp - mean) ** 2).sum() / m)
        adv[g0:g0 + m] = (grp - mean) / (std + delta)
    return adv


# ---------------------------------------------------------------------------- PPO
def path_logprob(path, tree, logits: np.ndarray, lse: np.ndarray):
    """log-probability, under the model whose logits/lse are given, of the accepted
    sequence: sum over its steps t of (logit of the accepted token at slot
    path_slot[t] of level t) - lse of that row.  Eq. 11 numerator terms."""
    R = path["path_len"].shape[0]
    out = np.zeros(R)
    for r in range(R):
        acc = 0.0
        for t in range(int(path["path_len"][r])):
            j = int(path["path_slot"][r, t])
            tok = int(tree["sel_tok"][r, int(path["path_node"][r, t])])
            acc += float(logits[r, t, j, tok]) - float(lse[r, t, j])
        out[r] = acc
    return out


def ppo_surrogate_fwd(path, tree, D_cur, d_lse, D_ref_on_cur, ref_lse, adv, m: int, eps: float = 0.2):
    """Eq. 11-12.  ratio s_i = exp((log M(S) - log M0(S)) / max(l_i, 1)); term_i =
    min(s_i A_i, clip(s_i, 1-eps, 1+eps) A_i); group loss = -(1/m) sum of terms;
    the K group losses are averaged.  `active` marks roots through which a
    gradient flows: l_i > 0 and the min picked the unclipped branch (A >= 0 and
    s <= 1+eps, or A < 0 and s >= 1-eps)."""
    adv = np.asarray(adv, dtype=np.float64)
    R = adv.shape[0]
    logM = path_logprob(path, tree, D_cur, d_lse)
    logM0 = path_logprob(path, tree, D_ref_on_cur, ref_lse)
    ratio = np.ones(R)
    term = np.zeros(R)
    active = np.zeros(R, dtype=np.int32)
    for r in range(R):
        l = int(path["path_len"][r])
        s = math.exp((logM[r] - logM0[r]) / max(l, 1))
        a = adv[r]
        clipped = max(1.0 - eps, min(s, 1.0 + eps))
        term[r] = min(s * a, clipped * a)
        ratio[r] = s
        passes = (s <= 1.0 + eps) if a >= 0 else (s >= 1.0 - eps)
        active[r] = 1 if (l > 0 and passes) else 0
    loss_group = np.array([-term[g0:g0 + m].sum() / m for g0 in range(0, R, m)])
    loss = float(loss_group.mean())
    return dict(logM=logM, logM0=logM0, ratio=ratio, term=term, active=active,
                loss_group=loss_group, loss=loss)


def ppo_surrogate_bwd(path, tree, fwd, D_cur, d_lse, adv, m: int, grad_scale: float = 1.0):
    """Gradient of grad_scale * loss w.r.t. the current draft logits.  Only the rows
    on the accepted path receive a gradient (the advantage and the discrete tree
    are constants): for step t < l_i of root i, with p = softmax of that row,
        G[i, t, v] = c_i (1[v = token_t] - p_v),
        c_i = grad_scale * (-A_i / (m K)) * active_i * s_i / max(l_i, 1),
    K = number of groups.  Rows t >= l_i are zero.  Returns grad_rows [R, d, V]
    fp64, grad_slot [R, d] (slot of level t the row belongs to, -1 if none) and
    coef [R]."""
    R, d, k, V = D_cur.shape
    K = R // m
    grad_rows = np.zeros((R, d, V))
    grad_slot = np.full((R, d), -1, dtype=np.int32)
    coef = np.zeros(R)
    for r in range(R):
        l = int(path["path_len"][r])
        c = grad_scale * (-float(adv[r]) / (m * K)) * int(fwd["active"][r]) * float(fwd["ratio"][r]) / max(l, 1)
        coef[r] = c
        for t in range(l):
            j = int(path["path_slot"][r, t])
            grad_slot[r, t] = j
            if c == 0.0:
                continue
            tok = int(tree["sel_tok"][r, int(path["path_node"][r, t])])
            p = np.exp(D_cur[r, t, j].astype(np.float64) - float(d_lse[r, t, j]))
            gvec = -c * p
            gvec[tok] += c
            grad_rows[r, t] = gvec
    return dict(grad_rows=grad_rows, grad_slot=grad_slot, coef=coef)


def ppo_surrogate_bwd_dh(bwd, W_vh: np.ndarray):
    """Fused LM-head variant: gradient of grad_scale * loss w.r.t. the current draft model's hidden
    states.  The logits of a slot are hidden . W^T, so by the chain rule the hidden state of the
    slot behind step t of root i receives
        dH[i, t, :] = sum_v G[i, t, v] W[v, :] = c_i (W[token_t, :] - sum_v p_v W[v, :]),
    with G, c_i and p of ppo_surrogate_bwd (`bwd` is its result).  Returns dh_rows [R, d, hidden]
    fp64 (zero where grad_slot is -1 or c_i = 0) and abs_bound [R, d, hidden] = sum_v |G| |W|, the
    scale against which a lower-precision contraction is judged."""
    G = bwd["grad_rows"]
    W64 = np.asarray(W_vh, dtype=np.float64)
    R, d, V = G.shape
    dh = np.zeros((R, d, W64.shape[1]))
    bound = np.zeros_like(dh)
    absW = np.abs(W64)
    for r in range(R):
        for t in range(d):
            if bwd["grad_slot"][r, t] >= 0 and bwd["coef"][r] != 0.0:
                dh[r, t] = G[r, t] @ W64
                bound[r, t] = np.abs(G[r, t]) @ absW
    return dict(dh_rows=dh, abs_bound=bound)


# --------------------------------------------------------------------- token-level loss
def token_loss(D: np.ndarray, T: np.ndarray, weight=None, grad_scale: float = 1.0):
    """Token-level loss of Eq. 13 / App. B.2: mean over the supervised positions of the cross-entropy
    H(p_T, p_M) = - sum_v p_T(v) log p_M(v) from the target's to the draft's next-token distribution
    under the same teacher-forced prefix, i.e. at the root slot (0, 0) of every root.  `weight`
    (0/1 per root) selects the supervised positions I(x); default all.  Returns loss_rows [R]
    (H per root, 0 where unsupervised), loss (mean over I), and grad [R, V] = d(grad_scale * loss) /
    d(draft logits of slot (0,0)) = grad_scale * w_r / |I| * (p_M - p_T)."""
    R, V = D.shape[0], D.shape[-1]
    w = np.ones(R) if weight is None else np.asarray(weight, dtype=np.float64)
    n = float(w.sum())
    loss_rows = np.zeros(R)
    grad = np.zeros((R, V))
    for r in range(R):
        x = D[r, 0, 0].astype(np.float64)
        t = T[r, 0, 0].astype(np.float64)
        _, lse_m = _row_lse(x)
        _, lse_t = _row_lse(t)
        p_t = np.exp(t - lse_t)
        p_m = np.exp(x - lse_m)
        fin = p_t > 0                       # 0 * log 0 := 0 (zero-probability target tokens add nothing)
        loss_rows[r] = w[r] * float(-(p_t[fin] * (x[fin] - lse_m)).sum())
        if n > 0:
            grad[r] = grad_scale * w[r] / n * (p_m - p_t)
    loss = float(loss_rows.sum() / n) if n > 0 else 0.0
    return dict(loss_rows=loss_rows, loss=loss, grad=grad)


# ------------------------------------------------------------------------ whole path
def full_path(D_cur, T_cur, D_ref, T_ref, *, k, d, g, m, eta=1.0, eps=0.2, delta=1e-6,
              grad_scale=1.0, reward_mode="lse", want_grad=True, logit_err=0.0, path_mode="greedy", U_cur=None,
              U_ref=None):
    """Algorithm 1, lines for one minibatch of R roots, composed from the steps
    above.  D_ref doubles as the reference model's logits at the current tree's
    slot coordinates (Eq. 11 denominator)."""
    out = {}
    for tag, D, T, U in (("cur", D_cur, T_cur, U_cur), ("ref", D_ref, T_ref, U_ref)):
        ds = draft_row_stats(D, k)
        pool = expand_tree(ds["top_tok"], ds["top_logp32"], d, k, ds["top_logp64"], ds["top_logit"], logit_err)
        tree = select_topg(pool, g, audit=True)
        ts = target_row_stats(T)
        rew = tree_reward(tree, T, ts["t_lse"], eta)
        if path_mode == "greedy":
            path = accepted_path(tree, ts["t_argmax"], d)
        elif path_mode == "max_l":
            path = max_l_path(tree, rew["node_cum"], d)
        else:
            path = sampled_path(tree, T, ts["t_lse"], U, d)
        out[tag] = dict(dstats=ds, pool=pool, tree=tree, tstats=ts, reward=rew, path=path)
    key = "reward_" + reward_mode
    adv = group_advantage(out["cur"]["reward"][key], out["ref"]["reward"][key], m, delta)
    cur = out["cur"]
    fwd = ppo_surrogate_fwd(cur["path"], cur["tree"], D_cur, cur["dstats"]["row_lse"],
                            D_ref, out["ref"]["dstats"]["row_lse"], adv, m, eps)
    out["adv"] = adv
    out["ppo"] = fwd
    if want_grad:
        out["bwd"] = ppo_surrogate_bwd(cur["path"], cur["tree"], fwd, D_cur,
                                       cur["dstats"]["row_lse"], adv, m, grad_scale)
    return out
