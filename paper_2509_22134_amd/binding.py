"""ctypes binding of libgto.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

GTO_BF16, GTO_F32 = 0, 1
GTO_REWARD_LSE, GTO_REWARD_MAX, GTO_REWARD_MEAN, GTO_REWARD_NODESUM = 0, 1, 2, 3
GTO_PATH_GREEDY, GTO_PATH_MAX_L, GTO_PATH_SAMPLED = 0, 1, 2
GTO_FLAG_GRAD_ZERO_FILL = 1
GTO_FLAG_TARGET_PRUNE = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgto.so")
_lib = None


class GtoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status}: {gto_strerror(status)}")


class gto_config(C.Structure):
    _fields_ = [("R", C.c_int32), ("d", C.c_int32), ("k", C.c_int32), ("g", C.c_int32), ("V", C.c_int32),
                ("dtype", C.c_int32), ("row_stride", C.c_int64), ("group_size", C.c_int32),
                ("reward_mode", C.c_int32), ("eta", C.c_float), ("eps", C.c_float), ("delta", C.c_float),
                ("grad_scale", C.c_float), ("flags", C.c_int32), ("path_mode", C.c_int32),
                ("waves_per_row", C.c_int32), ("fused_groups", C.c_int32), ("fused_layout", C.c_int32),
                ("reserved", C.c_int32)]

    @property
    def C(self):
        return self.k + (self.d - 1) * self.k * self.k

    @property
    def rho(self):
        return 1 + (self.d - 1) * self.k


def _ptr_struct(name, fields):
    return type(name, (C.Structure,), {"_fields_": [(f, C.c_void_p) for f in fields]})


_DRAFT = ("row_max", "row_lse", "top_tok", "top_logp")
_TARGET = ("t_max", "t_lse", "t_argmax")
_POOL = ("cand_tok", "cand_parent", "cand_depth", "cand_pslot", "cand_slot", "cand_score", "slot_cand")
_TREE = ("sel_cand", "sel_tok", "sel_parent", "sel_depth", "sel_pslot", "sel_slot", "sel_leaf", "sel_score", "n_sel",
         "slot_need")
_REWARD = ("node_q", "node_cum", "reward", "reward_aux", "n_leaves", "path_len", "path_node", "path_slot",
           "accept_u")   # accept_u: optional input of the sampled walk, put into the dict by the caller
_PPO = ("logM", "logM0", "ratio", "term", "active", "coef", "loss_group", "loss")
gto_draft_stats = _ptr_struct("gto_draft_stats", _DRAFT)
gto_target_stats = _ptr_struct("gto_target_stats", _TARGET)
gto_pool = _ptr_struct("gto_pool", _POOL)
gto_tree = _ptr_struct("gto_tree", _TREE)
gto_reward = _ptr_struct("gto_reward", _REWARD)
gto_ppo = _ptr_struct("gto_ppo", _PPO)


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2509_22134_amd.build` "
                           "(there is no CPU fallback)")
    L = C.CDLL(_LIB_PATH)
    P, VP, SZ = C.POINTER, C.c_void_p, C.c_size_t
    cfgp = P(gto_config)
    L.gto_version.restype = C.c_int
    L.gto_strerror.restype = C.c_char_p
    L.gto_strerror.argtypes = [C.c_int]
    L.gto_workspace_bytes.argtypes = [cfgp, P(SZ)]
    L.gto_draft_row_stats.argtypes = [cfgp, VP, P(gto_draft_stats), VP]
    L.gto_target_row_stats.argtypes = [cfgp, VP, P(gto_target_stats), VP]
    L.gto_expand_tree.argtypes = [cfgp, VP, P(gto_draft_stats), P(gto_pool), VP, SZ, VP]
    L.gto_expand_from_stats.argtypes = [cfgp, P(gto_draft_stats), P(gto_pool), VP]
    L.gto_select_topg.argtypes = [cfgp, P(gto_pool), P(gto_tree), VP]
    L.gto_tree_reward.argtypes = [cfgp, P(gto_tree), VP, P(gto_target_stats), P(gto_reward), VP, SZ, VP]
    L.gto_reward_from_stats.argtypes = [cfgp, P(gto_tree), VP, P(gto_target_stats), P(gto_reward), VP]
    L.gto_group_advantage.argtypes = [cfgp, VP, VP, VP, VP]
    L.gto_ppo_surrogate_fwd.argtypes = [cfgp, P(gto_tree), P(gto_reward), VP, P(gto_draft_stats), VP,
                                        P(gto_draft_stats), VP, P(gto_ppo), VP, SZ, VP]
    L.gto_ppo_surrogate_fwd_noalloc.argtypes = [cfgp, P(gto_tree), P(gto_reward), VP, P(gto_draft_stats), VP, VP,
                                                P(gto_ppo), VP]
    L.gto_ppo_surrogate_bwd.argtypes = [cfgp, P(gto_tree), P(gto_reward), P(gto_ppo), VP, P(gto_draft_stats),
                                        VP, VP, VP]
    L.gto_calibration_copy.argtypes = [VP, VP, SZ, VP]
    L.gto_token_loss_fwd.argtypes = [cfgp, VP, VP, P(gto_draft_stats), P(gto_target_stats), VP, VP, VP, VP, VP]
    L.gto_token_loss_bwd.argtypes = [cfgp, VP, VP, P(gto_draft_stats), P(gto_target_stats), VP, VP, C.c_float, VP, VP]
    L.gto_fused_token_loss_workspace_bytes.argtypes = [cfgp, C.c_int32, P(C.c_size_t)]
    L.gto_token_loss_fwd_fused.argtypes = [cfgp, VP, C.c_int32, VP, VP, P(gto_draft_stats), P(gto_target_stats), VP, VP,
                                           VP, VP, VP, SZ, VP]
    L.gto_token_loss_bwd_fused.argtypes = [cfgp, P(gto_draft_stats), P(gto_target_stats), VP, VP, C.c_float, VP, VP, SZ,
                                           VP]
    L.gto_fused_workspace_bytes.argtypes = [cfgp, C.c_int32, P(SZ)]
    L.gto_fused_draft_row_stats.argtypes = [cfgp, VP, C.c_int32, VP, P(gto_draft_stats), VP, VP, SZ, VP]
    L.gto_fused_target_row_stats.argtypes = [cfgp, VP, C.c_int32, VP, P(gto_target_stats), VP, SZ, VP]
    L.gto_expand_tree_fused.argtypes = [cfgp, VP, C.c_int32, VP, P(gto_draft_stats), P(gto_pool), VP, SZ, VP]
    L.gto_tree_reward_fused.argtypes = [cfgp, P(gto_tree), VP, C.c_int32, VP, P(gto_target_stats), P(gto_reward),
                                        VP, SZ, VP]
    L.gto_ppo_surrogate_bwd_fused.argtypes = [cfgp, P(gto_tree), P(gto_reward), P(gto_ppo), VP, C.c_int32, VP,
                                              P(gto_draft_stats), VP, VP, VP, SZ, VP]
    L.gto_ppo_surrogate_fwd_fused.argtypes = [cfgp, P(gto_tree), P(gto_reward), VP, VP, C.c_int32, VP,
                                              P(gto_draft_stats), P(gto_draft_stats), VP, P(gto_ppo), VP, SZ, VP]
    L.gto_fused_dh_workspace_bytes.argtypes = [cfgp, C.c_int32, P(C.c_size_t)]
    L.gto_ppo_surrogate_bwd_fused_dh.argtypes = [cfgp, P(gto_tree), P(gto_reward), P(gto_ppo), VP, C.c_int32, VP, VP,
                                                 P(gto_draft_stats), VP, VP, VP, SZ, VP]
    L.gto_profile_enable.argtypes = [C.c_int]
    L.gto_profile_read.argtypes = [P(C.c_char_p), P(C.c_int32), P(C.c_double), C.c_int]
    L.gto_profile_filter.argtypes = [C.c_char_p]
    for name in ("gto_workspace_bytes", "gto_draft_row_stats", "gto_target_row_stats", "gto_expand_tree",
                 "gto_expand_from_stats", "gto_select_topg", "gto_tree_reward", "gto_reward_from_stats",
                 "gto_group_advantage", "gto_ppo_surrogate_fwd", "gto_ppo_surrogate_bwd",
                 "gto_ppo_surrogate_fwd_noalloc",
                 "gto_profile_enable", "gto_profile_read", "gto_profile_filter", "gto_calibration_copy", "gto_token_loss_fwd", "gto_token_loss_bwd",
                 "gto_fused_workspace_bytes", "gto_fused_draft_row_stats", "gto_fused_target_row_stats",
                 "gto_expand_tree_fused", "gto_tree_reward_fused",
                 "gto_ppo_surrogate_fwd_fused", "gto_ppo_surrogate_bwd_fused",
                 "gto_fused_dh_workspace_bytes", "gto_ppo_surrogate_bwd_fused_dh",
                 "gto_fused_token_loss_workspace_bytes", "gto_token_loss_fwd_fused", "gto_token_loss_bwd_fused"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def make_config(*, R, d, k, g, V, dtype, row_stride=None, group_size=1, reward_mode=GTO_REWARD_LSE,
                eta=1.0, eps=0.2, delta=1e-6, grad_scale=1.0, flags=0, path_mode=0, waves_per_row=0,
                fused_groups=0, fused_layout=0) -> gto_config:
    if isinstance(dtype, torch.dtype):
        dtype = GTO_BF16 if dtype == torch.bfloat16 else GTO_F32
    return gto_config(R, d, k, g, V, dtype, V if row_stride is None else row_stride, group_size, reward_mode,
                      eta, eps, delta, grad_scale, flags, path_mode, waves_per_row, fused_groups, fused_layout, 0)


# ------------------------------------------------------------------ output containers (torch = memory only)
def _alloc(spec, device):
    # zero-filled so that entries the kernels never write (padding slots of level 0) are defined
    return {n: torch.zeros(shape, dtype=dt, device=device) for n, (shape, dt) in spec.items()}


def alloc_draft_stats(cfg, device) -> Dict[str, torch.Tensor]:
    s = (cfg.R, cfg.d, cfg.k)
    return _alloc({"row_max": (s, torch.float32), "row_lse": (s, torch.float32),
                   "top_tok": (s + (cfg.k,), torch.int32), "top_logp": (s + (cfg.k,), torch.float32)}, device)


def alloc_target_stats(cfg, device):
    s = (cfg.R, cfg.d, cfg.k)
    return _alloc({"t_max": (s, torch.float32), "t_lse": (s, torch.float32), "t_argmax": (s, torch.int32)}, device)


def alloc_pool(cfg, device):
    s = (cfg.R, cfg.C)
    spec = {n: (s, torch.int32) for n in _POOL[:5]}
    spec["cand_score"] = (s, torch.float32)
    spec["slot_cand"] = ((cfg.R, cfg.d, cfg.k), torch.int32)
    return _alloc(spec, device)


def alloc_tree(cfg, device):
    s = (cfg.R, cfg.g)
    spec = {n: (s, torch.int32) for n in _TREE[:7]}
    spec["sel_score"] = (s, torch.float32)
    spec["n_sel"] = ((cfg.R,), torch.int32)
    spec["slot_need"] = ((cfg.R, cfg.d, cfg.k), torch.int32)
    return _alloc(spec, device)


def alloc_reward(cfg, device):
    return _alloc({"node_q": ((cfg.R, cfg.g), torch.float32), "node_cum": ((cfg.R, cfg.g), torch.float32),
                   "reward": ((cfg.R,), torch.float32), "reward_aux": ((cfg.R, 4), torch.float32),
                   "n_leaves": ((cfg.R,), torch.int32), "path_len": ((cfg.R,), torch.int32),
                   "path_node": ((cfg.R, cfg.d), torch.int32), "path_slot": ((cfg.R, cfg.d), torch.int32)}, device)


def alloc_ppo(cfg, device):
    r = (cfg.R,)
    spec = {n: (r, torch.float32) for n in ("logM", "logM0", "ratio", "term", "coef")}
    spec["active"] = (r, torch.int32)
    spec["loss_group"] = ((cfg.R // max(cfg.group_size, 1),), torch.float32)
    spec["loss"] = ((1,), torch.float32)
    return _alloc(spec, device)


def _pack(struct_t, fields, tensors):
    if tensors is None:
        return None
    return struct_t(*[tensors[f].data_ptr() if tensors.get(f) is not None else None for f in fields])


def _ref(s):
    return C.byref(s) if s is not None else None


def _dp(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    elif isinstance(stream, torch.cuda.Stream):
        stream = stream.cuda_stream
    return C.c_void_p(stream)


def _check(status, where):
    if status != 0:
        raise GtoError(status, where)


# ------------------------------------------------------------------ entry points
def gto_version() -> int:
    return lib().gto_version()


def gto_strerror(status: int) -> str:
    return lib().gto_strerror(status).decode()


def gto_workspace_bytes(cfg) -> int:
    out = C.c_size_t(0)
    _check(lib().gto_workspace_bytes(C.byref(cfg), C.byref(out)), "gto_workspace_bytes")
    return out.value


def gto_draft_row_stats(cfg, draft_logits, stats, stream=None):
    s = _pack(gto_draft_stats, _DRAFT, stats)
    _check(lib().gto_draft_row_stats(C.byref(cfg), _dp(draft_logits), _ref(s), _stream(stream)), "gto_draft_row_stats")
    return stats


def gto_target_row_stats(cfg, target_logits, stats, stream=None):
    s = _pack(gto_target_stats, _TARGET, stats)
    _check(lib().gto_target_row_stats(C.byref(cfg), _dp(target_logits), _ref(s), _stream(stream)), "gto_target_row_stats")
    return stats


def gto_expand_tree(cfg, draft_logits, stats, pool, workspace=None, stream=None):
    s, p = _pack(gto_draft_stats, _DRAFT, stats), _pack(gto_pool, _POOL, pool)
    ws, wb = (_dp(workspace), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(lib().gto_expand_tree(C.byref(cfg), _dp(draft_logits), _ref(s), _ref(p), ws, wb, _stream(stream)),
           "gto_expand_tree")
    return stats, pool


def gto_expand_from_stats(cfg, stats, pool, stream=None):
    s, p = _pack(gto_draft_stats, _DRAFT, stats), _pack(gto_pool, _POOL, pool)
    _check(lib().gto_expand_from_stats(C.byref(cfg), _ref(s), _ref(p), _stream(stream)), "gto_expand_from_stats")
    return pool


def gto_select_topg(cfg, pool, tree, stream=None):
    p, t = _pack(gto_pool, _POOL, pool), _pack(gto_tree, _TREE, tree)
    _check(lib().gto_select_topg(C.byref(cfg), _ref(p), _ref(t), _stream(stream)), "gto_select_topg")
    return tree


def gto_tree_reward(cfg, tree, target_logits, stats, reward, workspace=None, stream=None):
    t, s, w = _pack(gto_tree, _TREE, tree), _pack(gto_target_stats, _TARGET, stats), _pack(gto_reward, _REWARD, reward)
    ws, wb = (_dp(workspace), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(lib().gto_tree_reward(C.byref(cfg), _ref(t), _dp(target_logits), _ref(s), _ref(w), ws, wb, _stream(stream)),
           "gto_tree_reward")
    return stats, reward


def gto_reward_from_stats(cfg, tree, target_logits, stats, reward, stream=None):
    t, s, w = _pack(gto_tree, _TREE, tree), _pack(gto_target_stats, _TARGET, stats), _pack(gto_reward, _REWARD, reward)
    _check(lib().gto_reward_from_stats(C.byref(cfg), _ref(t), _dp(target_logits), _ref(s), _ref(w), _stream(stream)),
           "gto_reward_from_stats")
    return reward


def gto_group_advantage(cfg, reward_cur, reward_ref, adv, stream=None):
    _check(lib().gto_group_advantage(C.byref(cfg), _dp(reward_cur), _dp(reward_ref), _dp(adv), _stream(stream)),
           "gto_group_advantage")
    return adv


def gto_ppo_surrogate_fwd(cfg, tree_cur, path_cur, draft_logits_cur, draft_stats_cur, ref_logits_on_cur,
                          ref_stats, adv, out, workspace=None, stream=None):
    t, w = _pack(gto_tree, _TREE, tree_cur), _pack(gto_reward, _REWARD, path_cur)
    ds, rs = _pack(gto_draft_stats, _DRAFT, draft_stats_cur), _pack(gto_draft_stats, _DRAFT, ref_stats)
    o = _pack(gto_ppo, _PPO, out)
    ws, wb = (_dp(workspace), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(lib().gto_ppo_surrogate_fwd(C.byref(cfg), _ref(t), _ref(w), _dp(draft_logits_cur), _ref(ds),
                                       _dp(ref_logits_on_cur), _ref(rs), _dp(adv), _ref(o), ws, wb, _stream(stream)),
           "gto_ppo_surrogate_fwd")
    return out


def gto_ppo_surrogate_fwd_noalloc(cfg, tree_cur, path_cur, draft_logits_cur, draft_stats_cur, ref_logits_on_cur,
                                  adv, out, stream=None):
    t, w = _pack(gto_tree, _TREE, tree_cur), _pack(gto_reward, _REWARD, path_cur)
    ds, o = _pack(gto_draft_stats, _DRAFT, draft_stats_cur), _pack(gto_ppo, _PPO, out)
    _check(lib().gto_ppo_surrogate_fwd_noalloc(C.byref(cfg), _ref(t), _ref(w), _dp(draft_logits_cur), _ref(ds),
                                               _dp(ref_logits_on_cur), _dp(adv), _ref(o), _stream(stream)),
           "gto_ppo_surrogate_fwd_noalloc")
    return out


def gto_ppo_surrogate_bwd(cfg, tree_cur, path_cur, fwd, draft_logits_cur, draft_stats_cur, grad_rows, grad_slot,
                          stream=None):
    t, w = _pack(gto_tree, _TREE, tree_cur), _pack(gto_reward, _REWARD, path_cur)
    f, ds = _pack(gto_ppo, _PPO, fwd), _pack(gto_draft_stats, _DRAFT, draft_stats_cur)
    _check(lib().gto_ppo_surrogate_bwd(C.byref(cfg), _ref(t), _ref(w), _ref(f), _dp(draft_logits_cur), _ref(ds),
                                       _dp(grad_rows), _dp(grad_slot), _stream(stream)), "gto_ppo_surrogate_bwd")
    return grad_rows, grad_slot


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _dp(workspace), workspace.numel() * workspace.element_size()


def gto_fused_workspace_bytes(cfg, hidden_dim: int) -> int:
    out = C.c_size_t(0)
    _check(lib().gto_fused_workspace_bytes(C.byref(cfg), hidden_dim, C.byref(out)), "gto_fused_workspace_bytes")
    return out.value


def gto_fused_draft_row_stats(cfg, hidden, w_vh, stats, workspace, top_logit=None, stream=None):
    s = _pack(gto_draft_stats, _DRAFT, stats)
    ws, wb = _ws(workspace)
    _check(lib().gto_fused_draft_row_stats(C.byref(cfg), _dp(hidden), hidden.shape[-1], _dp(w_vh), _ref(s),
                                           _dp(top_logit), ws, wb, _stream(stream)), "gto_fused_draft_row_stats")
    return stats


def gto_fused_target_row_stats(cfg, hidden, w_vh, stats, workspace, stream=None):
    s = _pack(gto_target_stats, _TARGET, stats)
    ws, wb = _ws(workspace)
    _check(lib().gto_fused_target_row_stats(C.byref(cfg), _dp(hidden), hidden.shape[-1], _dp(w_vh), _ref(s),
                                            ws, wb, _stream(stream)), "gto_fused_target_row_stats")
    return stats


def gto_expand_tree_fused(cfg, hidden, w_draft_vh, stats, pool, workspace, stream=None):
    s, p = _pack(gto_draft_stats, _DRAFT, stats), _pack(gto_pool, _POOL, pool)
    ws, wb = _ws(workspace)
    _check(lib().gto_expand_tree_fused(C.byref(cfg), _dp(hidden), hidden.shape[-1], _dp(w_draft_vh), _ref(s), _ref(p),
                                       ws, wb, _stream(stream)), "gto_expand_tree_fused")
    return stats, pool


def gto_tree_reward_fused(cfg, tree, hidden, w_target_vh, stats, reward, workspace, stream=None):
    t, s, w = _pack(gto_tree, _TREE, tree), _pack(gto_target_stats, _TARGET, stats), _pack(gto_reward, _REWARD, reward)
    ws, wb = _ws(workspace)
    _check(lib().gto_tree_reward_fused(C.byref(cfg), _ref(t), _dp(hidden), hidden.shape[-1], _dp(w_target_vh), _ref(s),
                                       _ref(w), ws, wb, _stream(stream)), "gto_tree_reward_fused")
    return stats, reward


def gto_ppo_surrogate_fwd_fused(cfg, tree_cur, path_cur, hidden_cur, hidden_ref_on_cur, w_draft_vh, draft_stats_cur,
                                ref_stats, adv, out, workspace, stream=None):
    t, w = _pack(gto_tree, _TREE, tree_cur), _pack(gto_reward, _REWARD, path_cur)
    ds, rs = _pack(gto_draft_stats, _DRAFT, draft_stats_cur), _pack(gto_draft_stats, _DRAFT, ref_stats)
    o = _pack(gto_ppo, _PPO, out)
    ws, wb = _ws(workspace)
    _check(lib().gto_ppo_surrogate_fwd_fused(C.byref(cfg), _ref(t), _ref(w), _dp(hidden_cur), _dp(hidden_ref_on_cur),
                                             hidden_cur.shape[-1], _dp(w_draft_vh), _ref(ds), _ref(rs), _dp(adv),
                                             _ref(o), ws, wb, _stream(stream)), "gto_ppo_surrogate_fwd_fused")
    return out


def gto_ppo_surrogate_bwd_fused(cfg, tree_cur, path_cur, fwd, hidden_cur, w_draft_vh, draft_stats_cur, grad_rows,
                                grad_slot, workspace, stream=None):
    t, w = _pack(gto_tree, _TREE, tree_cur), _pack(gto_reward, _REWARD, path_cur)
    f, ds = _pack(gto_ppo, _PPO, fwd), _pack(gto_draft_stats, _DRAFT, draft_stats_cur)
    ws, wb = _ws(workspace)
    _check(lib().gto_ppo_surrogate_bwd_fused(C.byref(cfg), _ref(t), _ref(w), _ref(f), _dp(hidden_cur),
                                             hidden_cur.shape[-1], _dp(w_draft_vh), _ref(ds), _dp(grad_rows),
                                             _dp(grad_slot), ws, wb, _stream(stream)), "gto_ppo_surrogate_bwd_fused")
    return grad_rows, grad_slot


def gto_fused_dh_workspace_bytes(cfg, hidden_dim: int) -> int:
    out = C.c_size_t(0)
    _check(lib().gto_fused_dh_workspace_bytes(C.byref(cfg), hidden_dim, C.byref(out)), "gto_fused_dh_workspace_bytes")
    return out.value


def gto_ppo_surrogate_bwd_fused_dh(cfg, tree_cur, path_cur, fwd, hidden_cur, w_draft_vh, w_draft_hv, draft_stats_cur,
                                   dh_rows, grad_slot, workspace, stream=None):
    t, w = _pack(gto_tree, _TREE, tree_cur), _pack(gto_reward, _REWARD, path_cur)
    f, ds = _pack(gto_ppo, _PPO, fwd), _pack(gto_draft_stats, _DRAFT, draft_stats_cur)
    ws, wb = _ws(workspace)
    _check(lib().gto_ppo_surrogate_bwd_fused_dh(C.byref(cfg), _ref(t), _ref(w), _ref(f), _dp(hidden_cur),
                                                hidden_cur.shape[-1], _dp(w_draft_vh), _dp(w_draft_hv), _ref(ds),
                                                _dp(dh_rows), _dp(grad_slot), ws, wb, _stream(stream)),
           "gto_ppo_surrogate_bwd_fused_dh")
    return dh_rows, grad_slot


def gto_token_loss_fwd(cfg, draft_logits, target_logits, draft_stats, target_stats, weight, loss_rows, loss,
                       inv_count, stream=None):
    ds, ts = _pack(gto_draft_stats, _DRAFT, draft_stats), _pack(gto_target_stats, _TARGET, target_stats)
    _check(lib().gto_token_loss_fwd(C.byref(cfg), _dp(draft_logits), _dp(target_logits), _ref(ds), _ref(ts),
                                    _dp(weight), _dp(loss_rows), _dp(loss), _dp(inv_count), _stream(stream)),
           "gto_token_loss_fwd")
    return loss_rows, loss


def gto_token_loss_bwd(cfg, draft_logits, target_logits, draft_stats, target_stats, weight, inv_count, grad_scale,
                       grad_rows0, stream=None):
    ds, ts = _pack(gto_draft_stats, _DRAFT, draft_stats), _pack(gto_target_stats, _TARGET, target_stats)
    _check(lib().gto_token_loss_bwd(C.byref(cfg), _dp(draft_logits), _dp(target_logits), _ref(ds), _ref(ts),
                                    _dp(weight), _dp(inv_count), float(grad_scale), _dp(grad_rows0), _stream(stream)),
           "gto_token_loss_bwd")
    return grad_rows0


def gto_fused_token_loss_workspace_bytes(cfg, hidden_dim: int) -> int:
    out = C.c_size_t(0)
    _check(lib().gto_fused_token_loss_workspace_bytes(C.byref(cfg), hidden_dim, C.byref(out)),
           "gto_fused_token_loss_workspace_bytes")
    return out.value


def gto_token_loss_fwd_fused(cfg, hidden, w_draft_vh, w_target_vh, draft_stats, target_stats, weight, loss_rows, loss,
                             inv_count, workspace, stream=None):
    ds, ts = _pack(gto_draft_stats, _DRAFT, draft_stats), _pack(gto_target_stats, _TARGET, target_stats)
    ws, wb = _ws(workspace)
    _check(lib().gto_token_loss_fwd_fused(C.byref(cfg), _dp(hidden), hidden.shape[-1], _dp(w_draft_vh), _dp(w_target_vh),
                                          _ref(ds), _ref(ts), _dp(weight), _dp(loss_rows), _dp(loss), _dp(inv_count),
                                          ws, wb, _stream(stream)), "gto_token_loss_fwd_fused")
    return loss_rows, loss


def gto_token_loss_bwd_fused(cfg, draft_stats, target_stats, weight, inv_count, grad_scale, grad_rows0, workspace,
                             stream=None):
    ds, ts = _pack(gto_draft_stats, _DRAFT, draft_stats), _pack(gto_target_stats, _TARGET, target_stats)
    ws, wb = _ws(workspace)
    _check(lib().gto_token_loss_bwd_fused(C.byref(cfg), _ref(ds), _ref(ts), _dp(weight), _dp(inv_count),
                                          float(grad_scale), _dp(grad_rows0), ws, wb, _stream(stream)),
           "gto_token_loss_bwd_fused")
    return grad_rows0


def gto_calibration_copy(src, dst, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib().gto_calibration_copy(_dp(src), _dp(dst), nbytes, _stream(stream)), "gto_calibration_copy")
    return dst


def gto_profile_enable(on: bool) -> None:
    _check(lib().gto_profile_enable(1 if on else 0), "gto_profile_enable")


def gto_profile_filter(kernel_name=None) -> None:
    _check(lib().gto_profile_filter(kernel_name.encode() if kernel_name else None), "gto_profile_filter")


def gto_profile_read(cap: int = 32):
    names = (C.c_char_p * cap)()
    launches = (C.c_int32 * cap)()
    total = (C.c_double * cap)()
    n = lib().gto_profile_read(names, launches, total, cap)
    if n < 0:
        raise GtoError(n, "gto_profile_read")
    return {names[i].decode(): (int(launches[i]), float(total[i])) for i in range(n)}
