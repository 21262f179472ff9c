"""Independent brute-force statements used to pin the oracle (CPU only, tiny inputs).

Written in probability space with explicit token-path tuples, full Python sorts and
recursion, so that it shares neither structure nor arithmetic with oracle/gto_oracle.py
(which works in log space on flat pool indices).  Inputs are chosen by the tests so
that ranking gaps are far above rounding, hence fp32-vs-fp64 keys cannot matter.
"""
import itertools
import math

import numpy as np


def softmax64(x):
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def build_tree(D_root, k, d, g):
    """D_root: [d, k, V] logits of one root.  Returns (kept, expanded_slot) where kept is
    a list of token-path tuples in kept order with their confidences, and expanded_slot
    maps an expanded path tuple to its (level, slot)."""
    V = D_root.shape[-1]
    expanded = {(): (0, 0)}
    conf = {(): 1.0}
    candidates = []   # (path, confidence, creation order)
    frontier = [()]
    order_no = 0
    for level in range(d):
        children = []
        for node in frontier:
            lvl, slot = expanded[node]
            p = softmax64(D_root[lvl, slot])
            toks = sorted(range(V), key=lambda v: (-p[v], v))[:k]
            for t in toks:
                child = node + (t,)
                conf[child] = conf[node] * p[t]
                children.append((child, conf[child], order_no))
                order_no += 1
        candidates.extend(children)
        if level + 1 < d:
            best = sorted(children, key=lambda c: (-c[1], c[2]))[:k] if level > 0 else children
            frontier = [c[0] for c in best]
            for j, c in enumerate(best):
                expanded[c[0]] = (level + 1, j)
    kept = sorted(candidates, key=lambda c: (-c[1], c[2]))[:g]
    return [(c[0], c[1]) for c in kept], expanded


def expected_accept_len_recursive(kept_paths, expanded, T_root):
    """E(n) = sum over kept children c of n of T(c | n) * (1 + E(c))."""
    kept = set(kept_paths)

    def E(node):
        if node not in expanded:
            return 0.0
        lvl, slot = expanded[node]
        p = softmax64(T_root[lvl, slot])
        tot = 0.0
        for c in kept:
            if len(c) == len(node) + 1 and c[:-1] == node:
                tot += p[c[-1]] * (1.0 + E(c))
        return tot
    return E(())


def expected_accept_len_enumerate(kept_paths, expanded, T_root, d):
    """Sum over ALL V^d target roll-outs of P(roll-out) * (longest prefix that is a kept
    node).  Contexts that are not expanded nodes get a uniform distribution (the accepted
    length is already decided there)."""
    kept = set(kept_paths)
    V = T_root.shape[-1]
    tot = 0.0
    for seq in itertools.product(range(V), repeat=d):
        prob = 1.0
        acc = 0
        alive = True
        for j in range(d):
            ctx = seq[:j]
            if ctx in expanded:
                lvl, slot = expanded[ctx]
                p = softmax64(T_root[lvl, slot])[seq[j]]
            else:
                p = 1.0 / V
            prob *= p
            if alive and seq[:j + 1] in kept:
                acc = j + 1
            else:
                alive = False
        tot += prob * acc
    return tot


def sequence_lengths(kept_paths, expanded, T_root):
    """Eq. 3-4 per root-to-leaf sequence: dict leaf path -> L."""
    kept = set(kept_paths)
    leaves = [p for p in kept if not any(len(c) == len(p) + 1 and c[:-1] == p for c in kept)]
    out = {}
    for leaf in leaves:
        L = 0.0
        prefix = 1.0
        for j in range(len(leaf)):
            lvl, slot = expanded[leaf[:j]]
            prefix *= softmax64(T_root[lvl, slot])[leaf[j]]
            L += prefix
        out[leaf] = L
    return out


def greedy_accept(kept_paths, expanded, T_root, d):
    kept = set(kept_paths)
    node = ()
    while len(node) < d and node in expanded:
        lvl, slot = expanded[node]
        row = np.asarray(T_root[lvl, slot], dtype=np.float64)
        tok = min(v for v in range(len(row)) if row[v] == row.max())
        if node + (tok,) not in kept:
            break
        node = node + (tok,)
    return node


def oracle_paths(pool, tree, r):
    """Token-path tuple of every kept node of root r, from the oracle's flat arrays."""
    n = int(tree["n_sel"][r])
    paths = []
    for i in range(n):
        toks = []
        j = i
        while j >= 0:
            toks.append(int(tree["sel_tok"][r, j]))
            j = int(tree["sel_parent"][r, j])
        paths.append(tuple(reversed(toks)))
    return paths
