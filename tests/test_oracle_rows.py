"""Pins for the oracle's row statistics (Fig. 1 caption: per-node top-k token probabilities)."""
import numpy as np
import pytest
import scipy.special as sp

from oracle import gto_oracle as O


def _rand(R, d, k, V, seed, quant=None):
    rng = np.random.default_rng(seed)
    x = rng.normal(0, 2, size=(R, d, k, V))
    if quant:
        x = np.round(x / quant) * quant     # force many exact ties, as bf16 storage does
    return x


@pytest.mark.parametrize("quant", [None, 0.5])
def test_topk_matches_python_sort_and_scipy(quant):
    R, d, k, V = 3, 3, 4, 57
    D = _rand(R, d, k, V, 1, quant)
    st = O.draft_row_stats(D, k)
    for r in range(R):
        for (l, j) in O.used_slots(d, k):
            row = D[r, l, j]
            want = sorted(range(V), key=lambda v: (-row[v], v))[:k]
            assert st["top_tok"][r, l, j].tolist() == want
            assert st["row_max"][r, l, j] == row.max()
            np.testing.assert_allclose(st["row_lse"][r, l, j], sp.logsumexp(row), rtol=1e-14)
            np.testing.assert_allclose(st["top_logp64"][r, l, j], sp.log_softmax(row)[want], rtol=1e-12, atol=1e-13)
            assert st["top_logp32"].dtype == np.float32
    # padding slots of level 0 are never touched
    assert np.isnan(st["row_lse"][:, 0, 1:]).all()


def test_softmax_mass_and_uniform_closed_form():
    V, k = 64, 4
    D = np.zeros((1, 2, k, V))
    st = O.draft_row_stats(D, k)
    np.testing.assert_allclose(st["row_lse"][0, 0, 0], np.log(V), rtol=1e-15)
    np.testing.assert_allclose(st["top_logp64"][0, 1, 2], -np.log(V) * np.ones(k), rtol=1e-15)
    assert st["top_tok"][0, 0, 0].tolist() == [0, 1, 2, 3]      # all equal: lowest ids first


def test_minus_inf_logits_have_zero_probability():
    V, k = 16, 3
    D = np.full((1, 1, k, V), -np.inf)
    D[0, 0, 0, 5] = np.log(0.75)
    D[0, 0, 0, 9] = np.log(0.25)
    st = O.draft_row_stats(D, k)
    assert st["top_tok"][0, 0, 0].tolist() == [5, 9, 0]
    np.testing.assert_allclose(st["row_lse"][0, 0, 0], 0.0, atol=1e-15)
    assert st["top_logp64"][0, 0, 0, 2] == -np.inf


def test_target_stats_argmax_lowest_id_and_lse():
    T = _rand(2, 3, 3, 40, 7, quant=1.0)
    st = O.target_row_stats(T)
    for r in range(2):
        for (l, j) in O.used_slots(3, 3):
            row = T[r, l, j]
            assert st["t_argmax"][r, l, j] == min(v for v in range(40) if row[v] == row.max())
            np.testing.assert_allclose(st["t_lse"][r, l, j], sp.logsumexp(row), rtol=1e-14)
            assert st["t_max"][r, l, j] == row.max()


def test_fused_logits_is_the_plain_dot_product_and_row_margins_flag_close_tops():
    rng = np.random.default_rng(3)
    R, d, k, Hd, V = 2, 2, 2, 5, 7
    H = rng.integers(-8, 8, size=(R, d, k, Hd)).astype(np.float32) / 4     # bf16-exact values
    W = rng.integers(-8, 8, size=(V, Hd)).astype(np.float32) / 8
    L = O.fused_logits(H, W)
    for r in range(R):
        for (l, j) in O.used_slots(d, k):
            for v in range(V):
                want = sum(float(H[r, l, j, h]) * float(W[v, h]) for h in range(Hd))
                assert L[r, l, j, v] == want                               # exact: small dyadic rationals
    assert not L[:, 0, 1:].any()
    X = np.zeros((1, 1, 2, 6))
    X[0, 0, 0] = [5.0, 4.0, 3.0, 2.9999, 0.0, -1.0]
    assert O.row_margins(X, 2, 1e-3)[0] == pytest.approx(1.0 / 2e-3)       # top-3 gaps: 1, 1
    assert O.row_margins(X, 3, 1e-3)[0] < 1.0                              # 3 vs 2.9999 is inside the error


def test_fp32_accumulation_error_bound_covers_simulated_fp32_sums():
    """The error granted to fp32-accumulated logits: simulate the accumulation (exact 16-product partial sums
    added to an fp32 accumulator, one rounding each) against the fp64 sum for many rows; the largest observed
    error must stay below the bound, and the bound must not be absurdly loose (within ~3x of the worst of
    20 000 samples at six standard deviations)."""
    import numpy as np
    from oracle import gto_oracle as O
    rng = np.random.default_rng(3)
    hidden, n = 2048, 20000
    h = rng.standard_normal((n, hidden)).astype(np.float32)
    wv = (rng.standard_normal((n, hidden)) * 0.05).astype(np.float32)
    prod = h.astype(np.float64) * wv.astype(np.float64)
    exact = prod.sum(axis=1)
    acc = np.zeros(n, dtype=np.float32)
    for s in range(0, hidden, 16):
        acc = (acc.astype(np.float64) + prod[:, s:s + 16].sum(axis=1)).astype(np.float32)
    err = np.abs(acc.astype(np.float64) - exact)
    bound = O.fp32_accumulation_error(hidden, float(np.abs(exact).max()))
    assert err.max() < bound
    assert bound < 6.0 * err.max()
