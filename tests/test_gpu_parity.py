"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Staged protocol
  stage 1  row kernels vs oracle: token ids, max, argmax bit-exact; lse / logp within tolerance.
  stage 2  the oracle's tree logic fed the GPU's own fp32 row statistics must reproduce every
           id, parent, slot, path index and fp32 score bit for bit (both sides then take each
           ranking decision in the same precision, the kernel's).
  stage 3  end to end vs the pure fp64 oracle: roots whose smallest fp64 ranking gap is above
           TAU must match exactly; roots below it are near ties (several results correct) and
           are covered by stage 2 only.  Floats within 1e-5 relative.
"""
import numpy as np
import pytest
import torch

import gto_synth as S
import gpu_util as U
import paper_2509_22134_amd as G
from oracle import gto_oracle as O
from paper_2509_22134_amd.pipeline import GtoPath

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _run_full(w, tens, device, row_stride=None, V=None, ref_stats_known=True, flags=0, reward_mode=0,
              grad_scale=0.5, path_mode=0):
    V = V or w.V
    path = GtoPath(R=tens["D_cur"].shape[0], d=w.d, k=w.k, g=w.g, V=V, dtype=w.torch_dtype, group_size=w.m,
                   device=device, row_stride=row_stride, eta=w.eta, eps=w.eps, delta=w.delta,
                   grad_scale=grad_scale, flags=flags, reward_mode=reward_mode, full_path=w.full_path,
                   path_mode=path_mode)
    if flags == 0 and w.full_path:
        path.grad_rows.fill_(7.0)       # untouched rows must stay untouched
    path.step(tens["D_cur"], tens["T_cur"], tens.get("D_ref"), tens.get("T_ref"), ref_stats_known=ref_stats_known)
    torch.cuda.synchronize()
    return path


def _compare_all(w, tens, path, V=None, roots=None, grad_scale=0.5, reward_key="reward_lse", flags=0):
    """Stages 1-3 for the roots in `roots` (default all), in this process."""
    V = V or w.V
    R = tens["D_cur"].shape[0]
    roots = list(range(R)) if roots is None else list(roots)
    sub = {n: U.logits_np(t[roots])[..., :V] for n, t in tens.items()}
    ora, n_ambig, n_clear, n_same = U.compare_trees(w, sub, U.bundle_np(path, roots, with_ppo=False))
    return ora, n_ambig


def _compare_ppo(w, tens, path, ora_unused=None, grad_scale=0.5, reward_key="reward_lse", flags=0, E=0.0):
    """Advantage, surrogate and gradient for the whole batch (groups need all roots), in this process."""
    V = path.cfg.V
    sub = {n: U.logits_np(t)[..., :V] for n, t in tens.items()}
    ora = O.full_path(sub["D_cur"], sub["T_cur"], sub["D_ref"], sub["T_ref"], k=w.k, d=w.d, g=w.g, m=w.m,
                      eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=grad_scale,
                      reward_mode=reward_key.replace("reward_", ""))
    bundle = U.bundle_np(path, grad="dense")
    same_tree, _, loss_group = U.compare_ppo(w, sub, bundle, ora, grad_scale=grad_scale, reward_key=reward_key,
                                             zero_fill=bool(flags & G.GTO_FLAG_GRAD_ZERO_FILL), untouched=7.0, E=E)
    # the batch loss is the mean of the group losses (Eq. 12 averaged over the K groups)
    np.testing.assert_allclose(path.ppo["loss"].cpu().numpy()[0], float(np.mean(loss_group)), rtol=1e-5 + 4 * E,
                               atol=1e-6 + 2 * w.d * E)
    return same_tree


# ------------------------------------------------------------------------------------ stage 1 sweeps
@pytest.mark.parametrize("waves", [1, 2, 4, 8])
@pytest.mark.parametrize("dtype,V,stride", [("bf16", 8192, 8192), ("bf16", 20011, 20016), ("bf16", 1000, 1000),
                                            ("bf16", 40, 40), ("f32", 1000, 1000), ("f32", 5003, 5004),
                                            ("f32", 9000, 9000)])
def test_row_kernels_match_oracle(gpu_device, dtype, V, stride, waves):
    _say(f"row kernels dtype={dtype} V={V} stride={stride} waves={waves}")
    R, d, k = 5, 3, 10
    w = S.scaled(S.CONFIGS["llama31_8b"], R=R, V=stride, d=d, k=k, g=20, dtype=dtype, n_peaks=8)
    tens = S.make_logits(w, gpu_device, want=("D_cur", "T_cur"))
    D, T = tens["D_cur"], tens["T_cur"]
    D[0, 1, 2, 5:V:7] = float("-inf")                  # zero-probability tokens
    D[1, 0, 0, :] = 1.5                                # a flat row: pure id tie-break
    T[1, 1, 1, :] = -2.0
    T[2, 2, 3, V - 1] = 40.0                           # argmax in the ragged tail
    D[2, 2, 1, V - 3:V] = 30.0                         # top entries in the ragged tail, tied
    if stride > V:
        D[..., V:] = 99.0                              # padding must never be read as data
        T[..., V:] = 99.0
    cfg = G.make_config(R=R, d=d, k=k, g=20, V=V, dtype=w.torch_dtype, row_stride=stride, waves_per_row=waves)
    ds = G.gto_draft_row_stats(cfg, D, U.alloc_poisoned(G.alloc_draft_stats, cfg, gpu_device))
    ts = G.gto_target_row_stats(cfg, T, U.alloc_poisoned(G.alloc_target_stats, cfg, gpu_device))
    torch.cuda.synchronize()
    Dn, Tn = U.logits_np(D)[..., :V], U.logits_np(T)[..., :V]
    U.check_row_stats(U.to_np(ds), O.draft_row_stats(Dn, k), Dn, k)
    U.check_target_stats(U.to_np(ts), O.target_row_stats(Tn))


def test_rows_with_fewer_than_k_finite_logits(gpu_device):
    _say("rows with < k finite logits")
    R, d, k, V = 2, 2, 4, 2048
    D = torch.full((R, d, k, V), float("-inf"), device=gpu_device, dtype=torch.bfloat16)
    D[..., 100] = 1.0
    D[..., 1900] = 0.5
    cfg = G.make_config(R=R, d=d, k=k, g=5, V=V, dtype=torch.bfloat16)
    ds = G.gto_draft_row_stats(cfg, D, G.alloc_draft_stats(cfg, gpu_device))
    torch.cuda.synchronize()
    Dn = U.logits_np(D)
    U.check_row_stats(U.to_np(ds), O.draft_row_stats(Dn, k), Dn, k)


def test_nan_rows_give_no_fault_and_leave_other_roots_alone(gpu_device):
    """The header's contract for a row that holds NaNs: unspecified values for that root, but every
    index written stays in range, the call completes, and roots of other groups are untouched.  Output
    buffers are poisoned first, so an entry that a kernel forgot to write shows up as a wild index."""
    _say("NaN rows: no fault, indices in range, other roots unchanged")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=9000, m=4)
    tens = S.make_logits(w, gpu_device)
    good = _run_full(w, tens, gpu_device)
    bad = {n: t.clone() for n, t in tens.items()}
    bad["D_cur"][1, 1, 2, :] = float("nan")            # a whole draft row
    bad["D_cur"][1, 0, 0, 100:4000] = float("nan")     # most of a root row
    bad["T_cur"][2, 1, 0, :] = float("nan")            # a whole target row
    bad["T_cur"][2, 0, 0, 17] = float("nan")           # a single entry
    bad["D_ref"][6, 2, 1, :] = float("nan")
    bad["T_ref"][6, 0, 0, :] = float("nan")
    for flags in (0, G.GTO_FLAG_TARGET_PRUNE):
        path = GtoPath(R=16, d=w.d, k=w.k, g=w.g, V=w.V, dtype=w.torch_dtype, group_size=w.m, device=gpu_device,
                       eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, flags=flags)
        U.poison_path(path)
        path.grad_rows.fill_(7.0)
        path.step(bad["D_cur"], bad["T_cur"], bad["D_ref"], bad["T_ref"])
        torch.cuda.synchronize()                       # completes: no fault, no hang
        used = torch.from_numpy(U.used_mask(16, w.d, w.k)).to(gpu_device)
        for tag in ("cur", "ref"):
            b = path.buf[tag]
            tt = b["dstats"]["top_tok"][used]
            assert bool(((tt >= 0) & (tt < w.V)).all()), tag
            tr, rw = b["tree"], b["reward"]
            assert bool((tr["n_sel"] == min(w.g, w.C)).all())
            assert bool(((tr["sel_tok"] >= 0) & (tr["sel_tok"] < w.V)).all())
            idx = torch.arange(w.g, device=gpu_device)[None, :]
            assert bool(((tr["sel_parent"] >= -1) & (tr["sel_parent"] < idx)).all())
            assert bool(((tr["sel_pslot"] >= 0) & (tr["sel_pslot"] < w.k)).all())
            assert bool(((tr["sel_slot"] >= -1) & (tr["sel_slot"] < w.k)).all())
            assert bool(((rw["path_len"] >= 0) & (rw["path_len"] <= w.d)).all())
            assert bool(((rw["path_node"] >= -1) & (rw["path_node"] < w.g)).all())
            assert bool(((rw["path_slot"] >= -1) & (rw["path_slot"] < w.k)).all())
            need = tr["slot_need"].bool() if flags else used
            ta = b["tstats"]["t_argmax"][need & used]
            assert bool(((ta >= 0) & (ta < w.V)).all()), tag
        assert bool(((path.grad_slot >= -1) & (path.grad_slot < w.k)).all())
        # roots 8..15 (groups 2 and 3) saw no NaN: identical to the clean run, bit for bit
        clean = slice(8, 16)
        for tag in ("cur", "ref"):
            for grp in ("pool", "tree", "reward"):
                for n, x in good.buf[tag][grp].items():
                    assert torch.equal(x[clean], path.buf[tag][grp][n][clean]), (flags, tag, grp, n)
        for n in ("logM", "logM0", "ratio", "term", "active"):
            assert torch.equal(good.ppo[n][clean], path.ppo[n][clean]), (flags, n)
        assert torch.equal(good.ppo["loss_group"][2:], path.ppo["loss_group"][2:])
        assert torch.equal(good.adv[clean], path.adv[clean])
        assert torch.equal(good.grad_slot[clean], path.grad_slot[clean])
        assert torch.equal(good.grad_rows[clean], path.grad_rows[clean])


# ------------------------------------------------------------------------------------ full path
def test_tiny_config_full_path(gpu_device):
    w = S.CONFIGS["tiny"]
    _say(f"full path config {w.name}")
    tens = S.make_logits(w, gpu_device)
    path = _run_full(w, tens, gpu_device)
    _, n_ambig = _compare_all(w, tens, path)
    _compare_ppo(w, tens, path)
    _say(f"  near-tie roots: {n_ambig}")


@pytest.mark.parametrize("name,R,V,kw", [
    ("llama31_8b", 16, 24000, {}),
    ("llama31_8b", 8, 20011, {"pad": 20016}),
    ("qwen3_8b", 16, 16384, {}),
    ("llama31_8b", 16, 12000, {"ref_sigma": None}),          # independent reference model
    ("tiny", 8, 1000, {"k": 1, "d": 5, "g": 3}),               # k = 1: greedy chain
    ("tiny", 8, 400, {"g": 500}),                              # g >= C: everything kept
    ("tiny", 8, 64, {"d": 1, "k": 8, "g": 4}),                 # single level
    ("vicuna13b", 16, 8000, {"full_path": True}),
    ("llama31_8b", 8, 8000, {"d": 7, "g": 50}),                # tree-configuration sweep of App. E:
    ("llama31_8b", 8, 8000, {"d": 8, "g": 70}),                # depth {6, 7, 8} x budget {50, 60, 70}
    ("llama31_8b", 8, 8000, {"d": 7, "g": 60}),                # the paper's own setting (App. B.1)
    ("tiny", 96, 300, {"m": 96}),                              # one advantage group over the batch (wave per group)
    ("tiny", 80, 300, {"m": 40}),                              # groups larger than 16, smaller than a wave
    ("tiny", 48, 300, {"m": 16}),                              # largest group still summed by one thread
])
def test_mid_size_full_path(gpu_device, name, R, V, kw):
    kw = dict(kw)
    pad = kw.pop("pad", None)
    w = S.scaled(S.CONFIGS[name], R=R, V=pad or V, **kw)
    _say(f"full path mid-size {name} R={R} V={V} {kw}")
    tens = S.make_logits(w, gpu_device)
    if pad:
        for t in tens.values():
            t[..., V:] = 77.0
    path = _run_full(w, tens, gpu_device, row_stride=pad, V=V)
    _, n_ambig = _compare_all(w, tens, path, V=V)
    _compare_ppo(w, tens, path)
    _say(f"  near-tie roots: {n_ambig}")
    assert n_ambig <= max(2, R // 4)


@pytest.mark.parametrize("k,d,g,V,dtype", [
    (64, 1, 64, 4096, "bf16"),          # widest branching (one wave's list holds 64 entries); a single level
    (63, 2, 4032, 1024, "f32"),         # largest pool two levels reach: C = 63 + 63^2 = 4032, every candidate kept
    (11, 32, 500, 512, "bf16"),         # deepest tree (32 levels): C = 11 + 31 * 121 = 3762
    (4, 2, 8, 2_000_000, "bf16"),       # a long row: 2 M logits (977 tiles of 2048, ragged tail of 1280)
])
def test_sizes_at_the_limits(gpu_device, k, d, g, V, dtype):
    """The limits the header states (k <= 64, d <= 32, C <= 4096) and a vocabulary far beyond the paper's."""
    _say(f"limits: k={k} d={d} g={g} V={V} {dtype}")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=2, V=V, k=k, d=d, g=g, m=2, dtype=dtype, n_peaks=min(32, V // 4))
    tens = S.make_logits(w, gpu_device)
    path = _run_full(w, tens, gpu_device)
    _compare_all(w, tens, path)
    _compare_ppo(w, tens, path)


def test_reference_stats_recomputed_in_workspace_and_zero_fill(gpu_device):
    _say("ppo fwd without reference stats; zero fill")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=9000)
    tens = S.make_logits(w, gpu_device)
    a = _run_full(w, tens, gpu_device)
    b = _run_full(w, tens, gpu_device, ref_stats_known=False, flags=G.GTO_FLAG_GRAD_ZERO_FILL)
    for n in ("ratio", "term", "loss", "coef", "logM0"):
        np.testing.assert_allclose(b.ppo[n].cpu().numpy(), a.ppo[n].cpu().numpy(), rtol=1e-6, atol=1e-7)
    assert torch.equal(a.grad_slot, b.grad_slot)
    _compare_ppo(w, tens, b, flags=G.GTO_FLAG_GRAD_ZERO_FILL)
    valid = (a.grad_slot >= 0)
    assert torch.equal(a.grad_rows[valid], b.grad_rows[valid])
    assert not b.grad_rows[~valid].any()


@pytest.mark.parametrize("mode,key", [(G.GTO_REWARD_MAX, "reward_max"), (G.GTO_REWARD_MEAN, "reward_mean"),
                                      (G.GTO_REWARD_NODESUM, "reward_nodesum")])
def test_reward_modes_and_no_debias(gpu_device, mode, key):
    _say(f"reward mode {key}")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=6000)
    tens = S.make_logits(w, gpu_device)
    path = _run_full(w, tens, gpu_device, reward_mode=mode)
    idx = ["reward_lse", "reward_max", "reward_mean", "reward_nodesum"].index(key)
    cur = path.buf["cur"]["reward"]
    assert torch.equal(cur["reward"], cur["reward_aux"][:, idx])
    _compare_ppo(w, tens, path, reward_key=key)
    adv = torch.empty_like(path.adv)
    G.gto_group_advantage(path.cfg, cur["reward"], None, adv)
    torch.cuda.synchronize()
    np.testing.assert_allclose(adv.cpu().numpy(), O.group_advantage(cur["reward"].cpu().numpy(), None, w.m, w.delta),
                               rtol=2e-6, atol=1e-6)


def test_target_row_pruning_changes_nothing_but_the_rows_read(gpu_device):
    _say("target-row pruning")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=16000)
    tens = S.make_logits(w, gpu_device)
    a = _run_full(w, tens, gpu_device)
    b = _run_full(w, tens, gpu_device, flags=G.GTO_FLAG_TARGET_PRUNE)
    b.grad_rows.copy_(a.grad_rows)                      # (rows without gradient are untouched in both)
    b.step(tens["D_cur"], tens["T_cur"], tens["D_ref"], tens["T_ref"])
    torch.cuda.synchronize()
    for tag in ("cur", "ref"):
        need = a.buf[tag]["tree"]["slot_need"].bool()
        assert torch.equal(need, b.buf[tag]["tree"]["slot_need"].bool())
        frac = need.float().sum().item() / (16 * w.rho)
        _say(f"  {tag}: {frac:.2f} of the target rows are needed")
        assert 0.05 < frac < 0.95 and bool(need[:, 0, 0].all()) and not bool(need[:, 0, 1:].any())
        for n, t in a.buf[tag]["tstats"].items():
            assert torch.equal(t[need], b.buf[tag]["tstats"][n][need]), n
            assert not b.buf[tag]["tstats"][n][~need].any(), n      # skipped rows were never written
        for grp in ("tree", "reward"):
            for n, t in a.buf[tag][grp].items():
                assert torch.equal(t, b.buf[tag][grp][n]), (tag, grp, n)
    for n, t in a.ppo.items():
        assert torch.equal(t, b.ppo[n]), n
    assert torch.equal(a.grad_slot, b.grad_slot) and torch.equal(a.grad_rows, b.grad_rows)
    _compare_all(w, tens, a)                              # slot_need itself is checked against the oracle here


def test_max_l_reading_of_the_longest_accepted_sequence(gpu_device):
    _say("path mode: branch with the largest expected acceptance length")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=12000)
    tens = S.make_logits(w, gpu_device)
    path = _run_full(w, tens, gpu_device, path_mode=G.GTO_PATH_MAX_L)
    Tn = {"cur": U.logits_np(tens["T_cur"]), "ref": U.logits_np(tens["T_ref"])}
    for tag in ("cur", "ref"):
        b = path.buf[tag]
        gd, gt, grew = U.to_np(b["dstats"]), U.to_np(b["tstats"]), U.to_np(b["reward"])
        pool2, tree2, rew2, _ = U.oracle_from_gpu_stats(gd, gt, Tn[tag], w.d, w.k, w.g, w.eta)
        path2 = O.max_l_path(tree2, rew2["node_cum"], w.d)
        for n in U.INT_PATH:
            assert np.array_equal(grew[n], path2[n]), (tag, n)
        assert (grew["path_len"] >= 1).all()              # a tree always has a best branch
    _compare_ppo(w, tens, path)


@pytest.mark.parametrize("name,R,V", [("tiny", 64, None), ("llama31_8b", 16, 12000)])
def test_sampled_reading_of_the_longest_accepted_sequence(gpu_device, name, R, V):
    _say(f"path mode: temperature-1 verification, {name}")
    w = S.scaled(S.CONFIGS[name], R=R, V=V or S.CONFIGS[name].V)
    tens = S.make_logits(w, gpu_device)
    un = S.make_uniforms(w, gpu_device)
    path = GtoPath(R=R, d=w.d, k=w.k, g=w.g, V=w.V, dtype=w.torch_dtype, group_size=w.m, device=gpu_device,
                   eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, path_mode=G.GTO_PATH_SAMPLED)
    path.grad_rows.fill_(7.0)
    path.step(tens["D_cur"], tens["T_cur"], tens["D_ref"], tens["T_ref"], accept_u=un)
    torch.cuda.synchronize()
    sub = {n: U.logits_np(t) for n, t in tens.items()}
    un_np = {tag: t.cpu().numpy().astype(np.float64) for tag, t in un.items()}
    ora = O.full_path(sub["D_cur"], sub["T_cur"], sub["D_ref"], sub["T_ref"], k=w.k, d=w.d, g=w.g, m=w.m, eta=w.eta,
                      eps=w.eps, delta=w.delta, want_grad=False, path_mode="sampled", U_cur=un_np["cur"],
                      U_ref=un_np["ref"])
    n_clear = 0
    lens = []
    for tag in ("cur", "ref"):
        b = path.buf[tag]
        gd, gt, grew = U.to_np(b["dstats"]), U.to_np(b["tstats"]), U.to_np(b["reward"])
        # the oracle's walk on the GPU's own fp32 statistics: every decision compares the same numbers
        pool2, tree2, rew2, _ = U.oracle_from_gpu_stats(gd, gt, sub["T_" + tag], w.d, w.k, w.g, w.eta)
        path2 = O.sampled_path(tree2, sub["T_" + tag], gt["t_lse"].astype(np.float64), un_np[tag], w.d)
        sure = path2["margin"] > 1e-9
        for n in U.INT_PATH:
            assert np.array_equal(grew[n][sure], path2[n][sure]), (tag, n)
        assert sure.sum() >= R - 1
        # against the pure fp64 oracle where neither the tree nor a decision is a near tie
        o = ora[tag]
        clear = (np.minimum(o["pool"]["min_margin"], o["tree"]["min_margin"]) >= U.TAU) & (o["path"]["margin"] > 1e-5)
        for n in U.INT_PATH:
            assert np.array_equal(grew[n][clear], o["path"][n][clear]), (tag, n)
        n_clear += int(clear.sum())
        lens.append(grew["path_len"])
    assert n_clear >= R                                   # most roots of both trees are compared end to end
    assert np.concatenate(lens).max() >= 1                # some walks accept something
    _compare_ppo(w, tens, path)


def test_kernel_timing_and_its_filter(gpu_device):
    """The measurement aid: with timing on, every kernel of a step is reported once per launch; with the
    filter set, only the named kernel is; the results of the step are the same either way."""
    _say("per-kernel timing and its filter")
    w = S.CONFIGS["tiny"]
    tens = S.make_logits(w, gpu_device)
    plain = _run_full(w, tens, gpu_device)
    G.gto_profile_read()                                   # drop whatever an earlier test left
    G.gto_profile_enable(True)
    try:
        timed = _run_full(w, tens, gpu_device)
        everything = G.gto_profile_read()
        G.gto_profile_filter("row_stats_draft")
        only = _run_full(w, tens, gpu_device)
        filtered = G.gto_profile_read()
    finally:
        G.gto_profile_filter(None)
        G.gto_profile_enable(False)
    assert {"row_stats_draft", "row_stats_target", "expand", "select_topg", "reward_path", "ppo_bwd"} <= set(everything)
    assert everything["row_stats_draft"][0] == 2 and everything["row_stats_draft"][1] > 0.0      # two trees per root
    assert set(filtered) == {"row_stats_draft"} and filtered["row_stats_draft"][0] == 2
    for other in (timed, only):
        assert torch.equal(plain.ppo["loss"], other.ppo["loss"]) and torch.equal(plain.grad_slot, other.grad_slot)
    _run_full(w, tens, gpu_device)
    assert G.gto_profile_read() == {}                      # timing off again: nothing recorded


def test_step_can_be_captured_in_a_hip_graph(gpu_device):
    """The library allocates nothing, clears nothing with memset and never synchronises, so one step can
    be recorded into a HIP graph.  Every replay (with the inputs changed in place and eager work and
    synchronisations in between) must reproduce the eager results bit for bit."""
    _say("graph capture of one step")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=9000)
    tens = S.make_logits(w, gpu_device)
    other = S.make_logits(S.scaled(w, seed=w.seed + 17), gpu_device)
    mk = lambda: GtoPath(R=16, d=w.d, k=w.k, g=w.g, V=w.V, dtype=w.torch_dtype, group_size=w.m, device=gpu_device,
                         eta=w.eta, eps=w.eps, delta=w.delta, grad_scale=0.5, flags=G.GTO_FLAG_GRAD_ZERO_FILL)
    eager, graphed = mk(), mk()
    buf = {n: t.clone() for n, t in tens.items()}                  # the graph reads these buffers
    graphed.step(buf["D_cur"], buf["T_cur"], buf["D_ref"], buf["T_ref"])     # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graphed.step(buf["D_cur"], buf["T_cur"], buf["D_ref"], buf["T_ref"])
    for it, src in enumerate((tens, other, tens, other)):
        for n in buf:
            buf[n].copy_(src[n])
        graph.replay()
        eager.step(src["D_cur"], src["T_cur"], src["D_ref"], src["T_ref"])
        torch.cuda.synchronize()
        for tag in ("cur", "ref"):
            for grp in ("dstats", "pool", "tree", "tstats", "reward"):
                for n, x in eager.buf[tag][grp].items():
                    if grp == "tstats":        # entries of slots without a kept child keep whatever they held
                        continue
                    assert torch.equal(x, graphed.buf[tag][grp][n]), (it, tag, grp, n)
        for n, x in eager.ppo.items():
            assert torch.equal(x, graphed.ppo[n]), (it, n)
        assert torch.equal(eager.adv, graphed.adv), it
        assert torch.equal(eager.grad_slot, graphed.grad_slot) and torch.equal(eager.grad_rows, graphed.grad_rows), it


def test_bitwise_deterministic(gpu_device):
    _say("determinism")
    w = S.scaled(S.CONFIGS["llama31_8b"], R=16, V=16000)
    tens = S.make_logits(w, gpu_device)
    a = _run_full(w, tens, gpu_device)
    b = _run_full(w, tens, gpu_device)
    for tag in ("cur", "ref"):
        for grp in ("dstats", "pool", "tree", "tstats", "reward"):
            for n, t in a.buf[tag][grp].items():
                if grp in ("dstats", "tstats"):
                    m = torch.from_numpy(U.used_mask(16, w.d, w.k)).to(t.device)
                    assert torch.equal(t[m], b.buf[tag][grp][n][m]), (tag, grp, n)
                else:
                    assert torch.equal(t, b.buf[tag][grp][n]), (tag, grp, n)
    for n, t in a.ppo.items():
        assert torch.equal(t, b.ppo[n]), n
    assert torch.equal(a.grad_slot, b.grad_slot)
    v = a.grad_slot >= 0
    assert torch.equal(a.grad_rows[v], b.grad_rows[v])


# ------------------------------------------------------------------------------------ token-level loss
@pytest.mark.parametrize("name,R,V,kw", [("llama31_8b", 16, 20000, {}), ("tiny", 8, 1000, {}),
                                         ("llama31_8b", 8, 5003, {"pad": 5008})])
def test_token_level_loss_fwd_bwd(gpu_device, name, R, V, kw):
    pad = kw.get("pad")
    w = S.scaled(S.CONFIGS[name], R=R, V=pad or V)
    _say(f"token-level loss {name} R={R} V={V}")
    tens = S.make_logits(w, gpu_device, want=("D_cur", "T_cur"))
    D, T = tens["D_cur"], tens["T_cur"]
    T[0, 0, 0, 7:V:3] = float("-inf")                       # zero-probability target tokens
    if pad:
        D[..., V:] = 50.0
        T[..., V:] = 50.0
    cfg = G.make_config(R=R, d=w.d, k=w.k, g=w.g, V=V, dtype=w.torch_dtype, row_stride=pad)
    ds = G.gto_draft_row_stats(cfg, D, G.alloc_draft_stats(cfg, gpu_device))
    ts = G.gto_target_row_stats(cfg, T, G.alloc_target_stats(cfg, gpu_device))
    weight = torch.ones(R, device=gpu_device)
    weight[1] = 0.0
    loss_rows = torch.empty(R, device=gpu_device); loss = torch.empty(1, device=gpu_device)
    inv = torch.empty(1, device=gpu_device); grad = torch.empty((R, V), device=gpu_device)
    Dn, Tn = U.logits_np(D)[..., :V], U.logits_np(T)[..., :V]
    for wt, wn in ((None, None), (weight, weight.cpu().numpy())):
        G.gto_token_loss_fwd(cfg, D, T, ds, ts, wt, loss_rows, loss, inv)
        G.gto_token_loss_bwd(cfg, D, T, ds, ts, wt, inv, 0.7, grad)
        torch.cuda.synchronize()
        ref = O.token_loss(Dn, Tn, wn, 0.7)
        np.testing.assert_allclose(loss_rows.cpu().numpy(), ref["loss_rows"], rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(loss.item(), ref["loss"], rtol=1e-5)
        g = grad.cpu().numpy()
        for r in range(R):
            scale = np.abs(ref["grad"][r]).max()
            assert np.abs(g[r] - ref["grad"][r]).max() <= 1e-5 * scale + 1e-12, r
