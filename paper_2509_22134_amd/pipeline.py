"""Orchestration of one pass of the GTO hot path over a batch of roots.

Buffers are allocated once (torch = device memory only); `step` issues the C-ABI calls in
the order of Algorithm 1 (build both trees, rewards, debias + standardise, surrogate forward,
gradient w.r.t. the current draft logits) on the current stream and returns without
synchronising.
"""
from __future__ import annotations

from typing import Dict, Optional

import torch

from . import binding as B


class GtoPath:
    def __init__(self, *, R, d, k, g, V, dtype, group_size, device, row_stride=None, eta=1.0, eps=0.2,
                 delta=1e-6, grad_scale=1.0, reward_mode=B.GTO_REWARD_LSE, flags=0, full_path=True,
                 want_grad=True, path_mode=0, waves_per_row=0):
        self.cfg = B.make_config(R=R, d=d, k=k, g=g, V=V, dtype=dtype, row_stride=row_stride,
                                 group_size=group_size, reward_mode=reward_mode, eta=eta, eps=eps,
                                 delta=delta, grad_scale=grad_scale, flags=flags, path_mode=path_mode,
                                 waves_per_row=waves_per_row)
        self.device = device
        self.full_path = full_path
        self.want_grad = want_grad and full_path
        tags = ("cur", "ref") if full_path else ("cur",)
        self.buf: Dict[str, Dict[str, Dict[str, torch.Tensor]]] = {}
        for tag in tags:
            self.buf[tag] = dict(dstats=B.alloc_draft_stats(self.cfg, device), pool=B.alloc_pool(self.cfg, device),
                                 tree=B.alloc_tree(self.cfg, device), tstats=B.alloc_target_stats(self.cfg, device),
                                 reward=B.alloc_reward(self.cfg, device))
        if full_path:
            self.adv = torch.empty((R,), dtype=torch.float32, device=device)
            self.ppo = B.alloc_ppo(self.cfg, device)
            self.workspace = torch.empty((B.gto_workspace_bytes(self.cfg),), dtype=torch.uint8, device=device)
        if self.want_grad:
            self.grad_rows = torch.empty((R, d, V), dtype=torch.float32, device=device)
            self.grad_slot = torch.empty((R, d), dtype=torch.int32, device=device)

    def build_and_score(self, tag: str, D: torch.Tensor, T: torch.Tensor):
        b = self.buf[tag]
        B.gto_expand_tree(self.cfg, D, b["dstats"], b["pool"])
        B.gto_select_topg(self.cfg, b["pool"], b["tree"])
        B.gto_tree_reward(self.cfg, b["tree"], T, b["tstats"], b["reward"])

    def step(self, D_cur, T_cur, D_ref: Optional[torch.Tensor] = None, T_ref: Optional[torch.Tensor] = None,
             ref_stats_known: bool = True, accept_u: Optional[Dict[str, torch.Tensor]] = None):
        """accept_u: {"cur": [R, d, k] fp32, "ref": ...} uniform numbers, needed by GTO_PATH_SAMPLED only."""
        for tag in self.buf:
            if accept_u:
                self.buf[tag]["reward"]["accept_u"] = accept_u[tag]
            else:
                self.buf[tag]["reward"].pop("accept_u", None)
        self.build_and_score("cur", D_cur, T_cur)
        if not self.full_path:
            return
        self.build_and_score("ref", D_ref, T_ref)
        cur, ref = self.buf["cur"], self.buf["ref"]
        B.gto_group_advantage(self.cfg, cur["reward"]["reward"], ref["reward"]["reward"], self.adv)
        B.gto_ppo_surrogate_fwd(self.cfg, cur["tree"], cur["reward"], D_cur, cur["dstats"], D_ref,
                                ref["dstats"] if ref_stats_known else None, self.adv, self.ppo,
                                workspace=self.workspace)
        if self.want_grad:
            B.gto_ppo_surrogate_bwd(self.cfg, cur["tree"], cur["reward"], self.ppo, D_cur, cur["dstats"],
                                    self.grad_rows, self.grad_slot)


class GtoFusedPath:
    """The same step with the logits produced on the fly from hidden states and LM heads
    (draft head for both draft models, target head for the target)."""

    def __init__(self, *, R, d, k, g, V, hidden, group_size, device, eta=1.0, eps=0.2, delta=1e-6,
                 grad_scale=1.0, reward_mode=B.GTO_REWARD_LSE, flags=0, want_grad=True, path_mode=0, want_dh=False,
                 fused_groups=0, fused_layout=0):
        self.cfg = B.make_config(R=R, d=d, k=k, g=g, V=V, dtype=B.GTO_BF16, group_size=group_size,
                                 reward_mode=reward_mode, eta=eta, eps=eps, delta=delta, grad_scale=grad_scale,
                                 flags=flags, path_mode=path_mode, fused_groups=fused_groups,
                                 fused_layout=fused_layout)
        self.hidden = hidden
        self.want_grad = want_grad
        self.buf = {}
        for tag in ("cur", "ref"):
            self.buf[tag] = dict(dstats=B.alloc_draft_stats(self.cfg, device), pool=B.alloc_pool(self.cfg, device),
                                 tree=B.alloc_tree(self.cfg, device), tstats=B.alloc_target_stats(self.cfg, device),
                                 reward=B.alloc_reward(self.cfg, device))
        self.adv = torch.empty((R,), dtype=torch.float32, device=device)
        self.ppo = B.alloc_ppo(self.cfg, device)
        self.workspace = torch.empty((B.gto_fused_workspace_bytes(self.cfg, hidden),), dtype=torch.uint8, device=device)
        if want_grad:
            self.grad_rows = torch.empty((R, d, V), dtype=torch.float32, device=device)
            self.grad_slot = torch.empty((R, d), dtype=torch.int32, device=device)
        self.want_dh = want_dh
        if want_dh:
            # gradient w.r.t. the hidden states instead of (or next to) the logits rows
            self.dh_rows = torch.empty((R, d, hidden), dtype=torch.float32, device=device)
            self.dh_slot = torch.empty((R, d), dtype=torch.int32, device=device)
            self.dh_workspace = torch.empty((B.gto_fused_dh_workspace_bytes(self.cfg, hidden),), dtype=torch.uint8,
                                            device=device)

    def build_and_score(self, tag, H, W_draft, W_target):
        b = self.buf[tag]
        B.gto_expand_tree_fused(self.cfg, H, W_draft, b["dstats"], b["pool"], self.workspace)
        B.gto_select_topg(self.cfg, b["pool"], b["tree"])
        B.gto_tree_reward_fused(self.cfg, b["tree"], H, W_target, b["tstats"], b["reward"], self.workspace)

    def step(self, H_cur, H_ref, W_draft, W_target, accept_u=None, W_draft_hv=None):
        """W_draft_hv: the draft head hidden-major ([hidden, V]), needed with want_dh only."""
        for tag in self.buf:
            if accept_u:
                self.buf[tag]["reward"]["accept_u"] = accept_u[tag]
            else:
                self.buf[tag]["reward"].pop("accept_u", None)
        self.build_and_score("cur", H_cur, W_draft, W_target)
        self.build_and_score("ref", H_ref, W_draft, W_target)
        cur, ref = self.buf["cur"], self.buf["ref"]
        B.gto_group_advantage(self.cfg, cur["reward"]["reward"], ref["reward"]["reward"], self.adv)
        B.gto_ppo_surrogate_fwd_fused(self.cfg, cur["tree"], cur["reward"], H_cur, H_ref, W_draft, cur["dstats"],
                                      ref["dstats"], self.adv, self.ppo, self.workspace)
        if self.want_grad:
            B.gto_ppo_surrogate_bwd_fused(self.cfg, cur["tree"], cur["reward"], self.ppo, H_cur, W_draft, cur["dstats"],
                                          self.grad_rows, self.grad_slot, self.workspace)
        if self.want_dh:
            B.gto_ppo_surrogate_bwd_fused_dh(self.cfg, cur["tree"], cur["reward"], self.ppo, H_cur, W_draft, W_draft_hv,
                                             cur["dstats"], self.dh_rows, self.dh_slot, self.dh_workspace)
