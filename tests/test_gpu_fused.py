"""GPU parity of the fused LM-head variant (logits = hidden . W^T on the matrix cores, never stored)
against the CPU oracle fed the fp64 logits of the same hidden states and heads.

The GPU accumulates the logits in fp32, so every logit carries an absolute error of up to E (checked
here against the oracle's fp64 value; see logit_error_bound).  Consequences, all derived from E:
row top-k / argmax are compared where the oracle's row margins are clear of E; tree decisions where
the oracle's audit (with E in its error budget) says so; floats within max(1e-5, 4 d E) relative.
The staged protocol is otherwise that of test_gpu_parity.py."""
import numpy as np
import pytest
import torch

import gto_synth as S
import gpu_util as U
import paper_2509_22134_amd as G
from oracle import gto_oracle as O
from paper_2509_22134_amd.pipeline import GtoFusedPath
from test_gpu_parity import _compare_ppo, _say

pytestmark = pytest.mark.gpu


logit_error_bound = U.logit_error_bound


def _oracle_logits(t, roots):
    H = {n: t[n][roots].float().cpu().numpy() for n in ("H_cur", "H_ref")}
    out = {}
    for head, tensors in (("W_draft", (("D_cur", "H_cur"), ("D_ref", "H_ref"))),
                          ("W_target", (("T_cur", "H_cur"), ("T_ref", "H_ref")))):
        W64 = t[head].double().cpu().numpy()              # converted once per head
        for name, hn in tensors:
            out[name] = O.fused_logits(H[hn], W64)
            _say(f"  oracle logits {name} done")
        del W64
    return out


def _run(w, t, device, flags=0, fused_groups=0, fused_layout=0):
    path = GtoFusedPath(R=t["H_cur"].shape[0], d=w.d, k=w.k, g=w.g, V=w.V, hidden=w.hidden, group_size=w.m,
                        device=device, eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, flags=flags,
                        fused_groups=fused_groups, fused_layout=fused_layout)
    if flags == 0:
        path.grad_rows.fill_(7.0)
    path.step(t["H_cur"], t["H_ref"], t["W_draft"], t["W_target"])
    torch.cuda.synchronize()
    return path


def _compare_fused(w, t, path, roots):
    L = _oracle_logits(t, roots)
    _, _, n_ambig, _, _ = U.compare_trees_fused(w, L, U.bundle_np(path, roots, with_ppo=False))
    return L, n_ambig


@pytest.mark.parametrize("R,d,k,g,hidden,V,corr", [
    (16, 3, 4, 12, 256, 3000, 0.9),        # ragged vocabulary tail, one row block with a tail
    (40, 3, 8, 20, 512, 5120, 0.9),        # two row blocks, list capacity 8
    (16, 4, 10, 30, 128, 2048, 0.8),       # k = 10: list capacity 16
    (16, 3, 4, 12, 256, 1024, 0.0),        # independent target head: mostly empty paths
])
def test_fused_full_path_matches_oracle(gpu_device, R, d, k, g, hidden, V, corr):
    w = S.FusedWorkload("case", R=R, V=V, k=k, d=d, g=g, m=8, hidden=hidden, h_scale=3.0, w_sigma=0.05,
                        w_corr=corr, ref_sigma=0.05)
    _say(f"fused full path R={R} d={d} k={k} g={g} hidden={hidden} V={V} corr={corr}")
    t = S.make_fused(w, gpu_device)
    path = _run(w, t, gpu_device)
    L, n_ambig = _compare_fused(w, t, path, list(range(R)))
    _say(f"  near-tie roots: {n_ambig}")
    _compare_ppo(w, L, path)
    assert n_ambig <= R            # of 2 R trees


def test_fused_sampled_walk(gpu_device):
    _say("fused: temperature-1 verification walk")
    w = S.FusedWorkload("case", R=24, V=3000, k=8, d=3, g=20, m=8, hidden=256, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.9, ref_sigma=0.05)
    t = S.make_fused(w, gpu_device)
    un = S.make_uniforms(w, gpu_device)
    path = GtoFusedPath(R=w.R, d=w.d, k=w.k, g=w.g, V=w.V, hidden=w.hidden, group_size=w.m, device=gpu_device,
                        eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, path_mode=G.GTO_PATH_SAMPLED)
    path.grad_rows.fill_(7.0)
    path.step(t["H_cur"], t["H_ref"], t["W_draft"], t["W_target"], accept_u=un)
    torch.cuda.synchronize()
    L = _oracle_logits(t, list(range(w.R)))
    E = logit_error_bound(w.hidden, max(float(np.abs(v).max()) for v in L.values()))
    total = 0
    for tag in ("cur", "ref"):
        b = path.buf[tag]
        gd, gt, grew = U.to_np(b["dstats"]), U.to_np(b["tstats"]), U.to_np(b["reward"])
        _, tree2, _, _ = U.oracle_from_gpu_stats(gd, gt, L["T_" + tag], w.d, w.k, w.g, w.eta)
        path2 = O.sampled_path(tree2, L["T_" + tag], gt["t_lse"].astype(np.float64),
                               un[tag].cpu().numpy().astype(np.float64), w.d)
        sure = path2["margin"] > 8 * E + 1e-6          # the GPU's token logits differ from the oracle's by up to E
        for n in U.INT_PATH:
            assert np.array_equal(grew[n][sure], path2[n][sure]), (tag, n)
        assert sure.sum() >= w.R - 2
        total += int(grew["path_len"].sum())
    assert total > 0
    _compare_ppo(w, L, path)


@pytest.mark.parametrize("nc", [1, 4])
def test_fused_row_statistics_when_the_maximum_moves_far(gpu_device, nc):
    """Logits that climb by tens and by hundreds along the vocabulary (and fall, for negative hidden
    states): the running sum of a row has to be re-referenced, or recomputed, when a new tile's
    maximum is far above the exponent reference the row carries.  All products and sums are exact in
    fp32 here (hidden states and head rows are constant vectors of bf16 values), so ids are compared
    exactly, ties included."""
    _say(f"fused row statistics with a moving maximum, chunks={nc}")
    R, d, k, hidden, V = 6, 2, 4, 64, 4096
    v = torch.arange(V, dtype=torch.float32)
    b = (v * (4.0 / V)).to(torch.bfloat16).float()        # slow climb: duplicates after rounding = ties
    b = b + (v >= 1024).float() * 1.0 + (v >= 2560).float() * 2.5     # jumps of 64 and 160 in the logits
    W = b[:, None].expand(V, hidden).to(torch.bfloat16).contiguous().to(gpu_device)
    scale = torch.tensor([1.0, -1.0, 0.5, -0.5, 2.0, 0.25])
    H = scale[:, None, None, None].expand(R, d, k, hidden).to(torch.bfloat16).contiguous().to(gpu_device)
    cfg = G.make_config(R=R, d=d, k=k, g=4, V=V, dtype=torch.bfloat16, fused_groups=nc)
    ws = torch.empty(G.gto_fused_workspace_bytes(cfg, hidden), dtype=torch.uint8, device=gpu_device)
    ds, ts = G.alloc_draft_stats(cfg, gpu_device), G.alloc_target_stats(cfg, gpu_device)
    G.gto_fused_draft_row_stats(cfg, H, W, ds, ws)
    G.gto_fused_target_row_stats(cfg, H, W, ts, ws)
    torch.cuda.synchronize()
    L = O.fused_logits(H.float().cpu().numpy(), W.float().cpu().numpy())
    od, ot = O.draft_row_stats(L, k), O.target_row_stats(L)
    gd, gt = U.to_np(ds), U.to_np(ts)
    m = U.used_mask(R, d, k)
    assert np.array_equal(gd["top_tok"][m], od["top_tok"][m])
    assert np.array_equal(gt["t_argmax"][m], ot["t_argmax"][m])
    assert np.array_equal(gd["row_max"][m], od["row_max"][m].astype(np.float32))
    np.testing.assert_allclose(gd["row_lse"][m], od["row_lse"][m], rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(gt["t_lse"][m], ot["t_lse"][m], rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(gd["top_logp"][m], od["top_logp64"][m], rtol=1e-5, atol=4e-5)


@pytest.mark.parametrize("R,d,k,g,hidden,V,flags", [
    (40, 3, 8, 20, 256, 3072, 0),                               # one row block of path rows
    (200, 3, 4, 12, 320, 2048, 0),                              # several row blocks, ragged hidden tile (320 = 256 + 64)
    (24, 4, 8, 24, 128, 4096, G.GTO_FLAG_GRAD_ZERO_FILL),
])
def test_fused_hidden_state_gradient(gpu_device, R, d, k, g, hidden, V, flags):
    """dH = G . W of the fused backward against the oracle's fp64 contraction.  Tolerance: the gradient
    row is staged as hi + lo bf16 (2^-17 relative per entry), built from fp32 logits (error E) and
    summed in fp32, all relative to sum_v |G| |W| (the oracle's abs_bound)."""
    w = S.FusedWorkload("case", R=R, V=V, k=k, d=d, g=g, m=8, hidden=hidden, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.9, ref_sigma=0.05)
    _say(f"fused dH R={R} d={d} k={k} hidden={hidden} V={V} flags={flags}")
    t = S.make_fused(w, gpu_device)
    W_hv = t["W_draft"].t().contiguous()
    path = GtoFusedPath(R=R, d=d, k=k, g=g, V=V, hidden=hidden, group_size=w.m, device=gpu_device, eta=w.eta,
                        eps=w.eps, delta=w.delta, grad_scale=0.5, flags=flags, want_dh=True)
    path.grad_rows.fill_(7.0)
    path.dh_rows.fill_(7.0)
    path.step(t["H_cur"], t["H_ref"], t["W_draft"], t["W_target"], W_draft_hv=W_hv)
    torch.cuda.synchronize()
    L = _oracle_logits(t, list(range(R)))
    E = logit_error_bound(hidden, max(float(np.abs(v).max()) for v in L.values()))
    # the oracle's backward on the GPU's own tree, path, advantage and ratio (as in _compare_ppo)
    cur = path.buf["cur"]
    g_tree, g_rew = U.to_np(cur["tree"]), U.to_np(cur["reward"])
    gpath = {n: g_rew[n] for n in U.INT_PATH}
    gp = U.to_np(path.ppo)
    g_adv = path.adv.cpu().numpy().astype(np.float64)
    od = O.draft_row_stats(L["D_cur"], k)
    f2 = dict(active=gp["active"], ratio=gp["ratio"].astype(np.float64))
    b2 = O.ppo_surrogate_bwd(gpath, g_tree, f2, L["D_cur"], od["row_lse"], g_adv, w.m, 0.5)
    want = O.ppo_surrogate_bwd_dh(b2, t["W_draft"].double().cpu().numpy())
    got = path.dh_rows.cpu().numpy()
    slot = path.dh_slot.cpu().numpy()
    assert np.array_equal(slot, path.grad_slot.cpu().numpy())
    live = (slot >= 0) & (b2["coef"] != 0)[:, None]
    assert live.sum() >= 8, "the case must exercise some rows"
    tol = (2.0 ** -17 + 2 * E + 1e-6) * want["abs_bound"] + 1e-30
    err = np.abs(got - want["dh_rows"])
    assert (err[live] <= tol[live]).all(), float((err[live] / tol[live]).max())
    assert np.abs(want["dh_rows"][live]).max() > 0
    dead = ~live
    if flags & G.GTO_FLAG_GRAD_ZERO_FILL:
        assert not got[slot < 0].any()
    else:
        assert (got[slot < 0] == 7.0).all()
    _say(f"  rows with a gradient: {int(live.sum())}, worst error / tolerance {float((err[live] / tol[live]).max()):.3f}")


@pytest.mark.parametrize("R,V,hidden", [(24, 3000, 256), (300, 1032, 128)])
def test_fused_token_level_loss(gpu_device, R, V, hidden):
    """Eq. 13 for the fused variant: the root-row logits come from the matrix cores (fp32, error E),
    so the cross-entropy and its gradient are compared within E-derived tolerances."""
    d, k, g = 3, 4, 12
    w = S.FusedWorkload("case", R=R, V=V, k=k, d=d, g=g, m=8, hidden=hidden, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.5, ref_sigma=0.05)
    _say(f"fused token-level loss R={R} V={V} hidden={hidden}")
    t = S.make_fused(w, gpu_device)
    cfg = G.make_config(R=R, d=d, k=k, g=g, V=V, dtype=torch.bfloat16, group_size=1)
    ws = torch.empty(G.gto_fused_workspace_bytes(cfg, hidden), dtype=torch.uint8, device=gpu_device)
    ds = G.gto_fused_draft_row_stats(cfg, t["H_cur"], t["W_draft"], G.alloc_draft_stats(cfg, gpu_device), ws)
    ts = G.gto_fused_target_row_stats(cfg, t["H_cur"], t["W_target"], G.alloc_target_stats(cfg, gpu_device), ws)
    tws = torch.empty(G.gto_fused_token_loss_workspace_bytes(cfg, hidden), dtype=torch.uint8, device=gpu_device)
    weight = torch.ones(R, device=gpu_device)
    weight[1] = 0.0
    loss_rows = torch.empty(R, device=gpu_device); loss = torch.empty(1, device=gpu_device)
    inv = torch.empty(1, device=gpu_device); grad = torch.empty((R, V), device=gpu_device)
    H = t["H_cur"].float().cpu().numpy()
    Dn = O.fused_logits(H, t["W_draft"].double().cpu().numpy())
    Tn = O.fused_logits(H, t["W_target"].double().cpu().numpy())
    E = logit_error_bound(hidden, max(float(np.abs(Dn).max()), float(np.abs(Tn).max())))
    for wt, wn in ((None, None), (weight, weight.cpu().numpy())):
        G.gto_token_loss_fwd_fused(cfg, t["H_cur"], t["W_draft"], t["W_target"], ds, ts, wt, loss_rows, loss, inv, tws)
        G.gto_token_loss_bwd_fused(cfg, ds, ts, wt, inv, 0.7, grad, tws)
        torch.cuda.synchronize()
        ref = O.token_loss(Dn, Tn, wn, 0.7)
        np.testing.assert_allclose(loss_rows.cpu().numpy(), ref["loss_rows"], rtol=1e-5, atol=8 * E + 2e-6)
        np.testing.assert_allclose(loss.item(), ref["loss"], rtol=1e-5, atol=8 * E + 2e-6)
        gq = grad.cpu().numpy()
        for r in range(R):
            scale = np.abs(ref["grad"][r]).max()
            assert np.abs(gq[r] - ref["grad"][r]).max() <= (1e-5 + 8 * E) * scale + 1e-12, r


def test_fused_step_can_be_captured_in_a_hip_graph(gpu_device):
    _say("fused: graph capture of one step")
    w = S.FusedWorkload("case", R=24, V=3072, k=8, d=3, g=20, m=8, hidden=256, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.9, ref_sigma=0.05)
    t = S.make_fused(w, gpu_device)
    t2 = S.make_fused(S.scaled(w, seed=w.seed + 3), gpu_device)
    mk = lambda: GtoFusedPath(R=w.R, d=w.d, k=w.k, g=w.g, V=w.V, hidden=w.hidden, group_size=w.m, device=gpu_device,
                              eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, flags=G.GTO_FLAG_GRAD_ZERO_FILL,
                              want_dh=True)
    eager, graphed = mk(), mk()
    buf = {n: x.clone() for n, x in t.items()}
    hv = buf["W_draft"].t().contiguous()
    graphed.step(buf["H_cur"], buf["H_ref"], buf["W_draft"], buf["W_target"], W_draft_hv=hv)    # warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graphed.step(buf["H_cur"], buf["H_ref"], buf["W_draft"], buf["W_target"], W_draft_hv=hv)
    for it, src in enumerate((t, t2, t)):
        for n in buf:
            buf[n].copy_(src[n])
        hv.copy_(src["W_draft"].t())
        graph.replay()
        eager.step(src["H_cur"], src["H_ref"], src["W_draft"], src["W_target"], W_draft_hv=src["W_draft"].t().contiguous())
        torch.cuda.synchronize()
        for tag in ("cur", "ref"):
            for grp in ("dstats", "pool", "tree", "tstats", "reward"):
                for n, x in eager.buf[tag][grp].items():
                    assert torch.equal(x, graphed.buf[tag][grp][n]), (it, tag, grp, n)
        for n, x in eager.ppo.items():
            assert torch.equal(x, graphed.ppo[n]), (it, n)
        assert torch.equal(eager.grad_slot, graphed.grad_slot) and torch.equal(eager.grad_rows, graphed.grad_rows), it
        assert torch.equal(eager.dh_slot, graphed.dh_slot) and torch.equal(eager.dh_rows, graphed.dh_rows), it


def test_fused_chunking_and_layout_do_not_change_results(gpu_device):
    _say("fused: launch geometry (groups, patch shape) invariance")
    w = S.FusedWorkload("case", R=24, V=4096, k=8, d=3, g=20, m=8, hidden=256, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.9, ref_sigma=0.05)
    t = S.make_fused(w, gpu_device)
    ref = _run(w, t, gpu_device)
    for nc, layout in ((1, 1), (3, 0), (8, 1), (16, 0)):
        other = _run(w, t, gpu_device, fused_groups=nc, fused_layout=layout)
        for tag in ("cur", "ref"):
            for grp in ("tree", "reward"):
                for n, x in ref.buf[tag][grp].items():
                    if x.dtype == torch.int32:
                        assert torch.equal(x, other.buf[tag][grp][n]), (nc, tag, grp, n)
        assert torch.equal(ref.grad_slot, other.grad_slot)
        v = ref.grad_slot >= 0
        torch.testing.assert_close(ref.grad_rows[v], other.grad_rows[v], rtol=1e-5, atol=1e-9)


def test_fused_target_pruning_changes_nothing_but_the_rows_multiplied(gpu_device):
    _say("fused: target-row pruning")
    w = S.FusedWorkload("case", R=40, V=3000, k=8, d=3, g=20, m=8, hidden=256, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.9, ref_sigma=0.05)
    t = S.make_fused(w, gpu_device)
    a = _run(w, t, gpu_device)
    b = _run(w, t, gpu_device, flags=G.GTO_FLAG_TARGET_PRUNE)
    for tag in ("cur", "ref"):
        need = a.buf[tag]["tree"]["slot_need"].bool()
        frac = need.float().sum().item() / (w.R * w.rho)
        _say(f"  {tag}: {frac:.2f} of the target rows are needed")
        assert 0.05 < frac < 0.95
        for n, x in a.buf[tag]["tstats"].items():
            assert torch.equal(x[need], b.buf[tag]["tstats"][n][need]), n
            assert not b.buf[tag]["tstats"][n][~need].any(), n
        for grp in ("tree", "reward"):
            for n, x in a.buf[tag][grp].items():
                assert torch.equal(x, b.buf[tag][grp][n]), (tag, grp, n)
    for n, x in a.ppo.items():
        assert torch.equal(x, b.ppo[n]), n
    v = a.grad_slot >= 0
    assert torch.equal(a.grad_slot, b.grad_slot) and torch.equal(a.grad_rows[v], b.grad_rows[v])


def test_fused_zero_fill(gpu_device):
    w = S.FusedWorkload("case", R=16, V=2048, k=4, d=3, g=12, m=8, hidden=128, h_scale=3.0, w_sigma=0.05,
                        w_corr=0.9, ref_sigma=0.05)
    t = S.make_fused(w, gpu_device)
    a = _run(w, t, gpu_device)
    b = _run(w, t, gpu_device, flags=G.GTO_FLAG_GRAD_ZERO_FILL)
    v = a.grad_slot >= 0
    assert torch.equal(a.grad_slot, b.grad_slot) and torch.equal(a.grad_rows[v], b.grad_rows[v])
    assert not b.grad_rows[~v].any() and bool((a.grad_rows[~v] == 7.0).all())
