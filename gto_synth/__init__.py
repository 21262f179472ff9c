"""Seeded synthetic logits for the GTO hot path.

This module only draws random inputs; it holds none of the method's arithmetic
(no softmax, no top-k, no tree logic).  Both the HIP path and the CPU oracle are
fed the tensors produced here: they are generated once (on the GPU when there is
one), rounded to the storage dtype, and the very same bits are copied to the host
for the oracle.

The tensors stand in for the logits a draft model, its frozen reference copy and
the target model would produce at the expanded nodes of a draft tree; the paper's
training corpora and evaluation suites are not available, so shapes follow the
model vocabularies and tree settings (k = 10, g = 60: App. B.1, B.3) and value
distributions follow the recipes below.

Layout of every tensor: [R, d, k, V], row-major; slot (l, j) is the distribution
at the j-th expanded node of level l, level 0 uses slot (0, 0) only.

Recipes
  gauss_plant_target   x ~ N(0, sigma^2); with probability p the target row gets
                       max(T_row)+1 written at argmax(D_row)         (tiny config)
  gauss_plant_shared   x ~ N(0, sigma^2); with probability p one seeded token
                       gets max(row)+1 in both the draft and the target row
  zipf_peaks           x ~ N(0, sigma^2) plus P seeded peak positions with
                       x[peak_i] += a - s*ln(i), i = 1..P (a Zipf(s) profile in
                       probability space); a target row reuses its draft row's
                       peak positions with probability p, else draws its own
Reference model: D_ref = round(D_cur before rounding + N(0, ref_sigma^2)) (a
perturbed copy, second seed) unless ref_sigma is None, in which case D_ref is an
independent draw from the second seed.  T_ref is always an independent draw from
the second seed that shares D_ref's planted structure with probability p.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch

BASE_SEED = 0x47544F00


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    R: int
    V: int
    k: int
    d: int
    g: int
    m: int
    dtype: str = "bf16"            # storage dtype of the logits: "bf16" | "f32"
    recipe: str = "zipf_peaks"
    sigma: float = 2.0
    p_agree: float = 0.7
    n_peaks: int = 32
    peak_a: float = 14.0
    peak_s: float = 1.1
    ref_sigma: Optional[float] = 0.125
    seed: int = BASE_SEED
    eta: float = 1.0
    eps: float = 0.2
    delta: float = 1e-6
    chunk_roots: int = 0           # >0: the harness processes this many roots per pass
    full_path: bool = True         # False: reward only (one tree per root)

    @property
    def rho(self) -> int:
        return 1 + (self.d - 1) * self.k

    @property
    def C(self) -> int:
        return self.k + (self.d - 1) * self.k * self.k

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


CONFIGS: Dict[str, Workload] = {
    "tiny": Workload("tiny", R=4, V=1000, k=4, d=3, g=10, m=4, dtype="f32",
                     recipe="gauss_plant_target", sigma=2.0, p_agree=0.6, seed=BASE_SEED + 1),
    "vicuna13b": Workload("vicuna13b", R=512, V=32000, k=10, d=6, g=60, m=8,
                          recipe="gauss_plant_shared", sigma=3.0, p_agree=0.7,
                          seed=BASE_SEED + 2, full_path=False),
    "llama31_8b": Workload("llama31_8b", R=1024, V=128256, k=10, d=6, g=60, m=8, seed=BASE_SEED + 3),
    "qwen3_8b": Workload("qwen3_8b", R=2048, V=151936, k=8, d=7, g=64, m=8,
                         seed=BASE_SEED + 4, chunk_roots=256),
}


def scaled(w: Workload, **kw) -> Workload:
    """Same recipe at another size (used by parity tests that need oracle-sized inputs)."""
    return dataclasses.replace(w, **kw)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def _noise(shape, sigma, device, seed):
    return torch.randn(shape, generator=_gen(device, seed), device=device, dtype=torch.float32) * sigma


def _coin(shape, p, device, seed):
    return torch.rand(shape, generator=_gen(device, seed), device=device) < p


def _positions(shape, V, device, seed):
    return torch.randint(0, V, shape, generator=_gen(device, seed), device=device, dtype=torch.int64)


def _peak_heights(w: Workload, device):
    i = torch.arange(1, w.n_peaks + 1, device=device, dtype=torch.float32)
    return w.peak_a - w.peak_s * torch.log(i)


def _set_top(X, tok, on):
    """Where `on`, write max(row)+1 at position `tok` of each row of X (in place)."""
    top = X.max(dim=-1, keepdim=True).values + 1.0
    X.scatter_(-1, tok, torch.where(on, top, X.gather(-1, tok)))


def _root_block(w: Workload, r0: int, r1: int, device, want):
    """Tensors for roots [r0, r1).  Seeds are derived per (tensor, first root of
    the block), so the block decomposition (`block_roots`) is part of the recipe."""
    n = r1 - r0
    shape = (n, w.d, w.k, w.V)
    rows = (n, w.d, w.k)
    s0 = w.seed * 1000003 + r0 * 101
    s1 = (w.seed + 1) * 1000003 + r0 * 101     # "second seed": reference model / tree
    perturbed = w.ref_sigma is not None
    D_cur = _noise(shape, w.sigma, device, s0 + 1)
    T_cur = _noise(shape, w.sigma, device, s0 + 2)
    T_ref = _noise(shape, w.sigma, device, s1 + 2)
    coin_cur = _coin(rows, w.p_agree, device, s0 + 5).unsqueeze(-1)
    coin_ref = _coin(rows, w.p_agree, device, s1 + 5).unsqueeze(-1)

    def ref_draft():
        if perturbed:
            return D_cur + _noise(shape, w.ref_sigma, device, s1 + 1)
        return _noise(shape, w.sigma, device, s1 + 1)

    if w.recipe == "zipf_peaks":
        h = _peak_heights(w, device).expand(*rows, w.n_peaks)
        pos_D = _positions((*rows, w.n_peaks), w.V, device, s0 + 3)
        pos_T = _positions((*rows, w.n_peaks), w.V, device, s0 + 4)
        D_cur.scatter_add_(-1, pos_D, h)
        T_cur.scatter_add_(-1, torch.where(coin_cur, pos_D, pos_T), h)
        D_ref = ref_draft()
        if perturbed:
            pos_Dr = pos_D
        else:
            pos_Dr = _positions((*rows, w.n_peaks), w.V, device, s1 + 3)
            D_ref.scatter_add_(-1, pos_Dr, h)
        pos_Tr = _positions((*rows, w.n_peaks), w.V, device, s1 + 4)
        T_ref.scatter_add_(-1, torch.where(coin_ref, pos_Dr, pos_Tr), h)
    elif w.recipe == "gauss_plant_shared":
        tok = _positions((*rows, 1), w.V, device, s0 + 3)
        _set_top(D_cur, tok, coin_cur)
        _set_top(T_cur, tok, coin_cur)
        D_ref = ref_draft()
        if perturbed:
            tok_r = tok
        else:
            tok_r = _positions((*rows, 1), w.V, device, s1 + 3)
            _set_top(D_ref, tok_r, coin_ref)
        _set_top(T_ref, tok_r, coin_ref)
    elif w.recipe == "gauss_plant_target":
        _set_top(T_cur, D_cur.argmax(dim=-1, keepdim=True), coin_cur)
        D_ref = ref_draft()
        _set_top(T_ref, D_ref.argmax(dim=-1, keepdim=True), coin_ref)
    else:
        raise ValueError(f"unknown recipe {w.recipe}")
    allv = {"D_cur": D_cur, "T_cur": T_cur, "D_ref": D_ref, "T_ref": T_ref}
    return {name: allv[name].to(w.torch_dtype) for name in want}


def block_roots(w: Workload) -> int:
    """Roots generated per block: bounded so that the fp32 staging of four tensors
    stays near 2 GiB."""
    per_root = w.d * w.k * w.V * 4 * 4
    return max(1, min(w.R, (2 << 30) // per_root))


def make_uniforms(w, device, seed_offset: int = 0) -> Dict[str, torch.Tensor]:
    """Uniform numbers in [0, 1) for the temperature-1 verification walk: one fp32 [R, d, k] tensor per
    tree ("cur", "ref"), drawn from the workload's seed (+ 7919 + seed_offset) on the CPU so that the
    bits do not depend on the device."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed + 7919 + seed_offset)
    out = {}
    for tag in ("cur", "ref"):
        out[tag] = torch.rand((w.R, w.d, w.k), generator=gen, dtype=torch.float32).to(device)
    return out


def make_logits(w: Workload, device, want=("D_cur", "T_cur", "D_ref", "T_ref"),
                roots: Optional[range] = None) -> Dict[str, torch.Tensor]:
    """Generate the requested tensors for `roots` (default: all R roots) on
    `device`.  Roots must start and end on block boundaries (or at R)."""
    device = torch.device(device)
    roots = roots if roots is not None else range(0, w.R)
    r_lo, r_hi = roots.start, roots.stop
    B = block_roots(w)
    assert r_lo % B == 0 and (r_hi % B == 0 or r_hi == w.R), "roots must align to generator blocks"
    n = r_hi - r_lo
    out = {name: torch.empty((n, w.d, w.k, w.V), dtype=w.torch_dtype, device=device) for name in want}
    for b0 in range(r_lo, r_hi, B):
        b1 = min(b0 + B, r_hi)
        blk = _root_block(w, b0, b1, device, want)
        for name in want:
            out[name][b0 - r_lo:b1 - r_lo] = blk[name]
        del blk
    return out


# ----------------------------------------------------------------------------- fused LM-head workload
@dataclasses.dataclass(frozen=True)
class FusedWorkload:
    """Hidden states and LM heads instead of logits: D = H . W_draft^T, T = H . W_target^T.
    H_cur ~ N(0, h_scale^2) (seed); H_ref = H_cur + N(0, ref_sigma^2) from the second seed (None: an
    independent draw); W_draft ~ N(0, w_sigma^2) (seed), W_target = corr * W_draft + sqrt(1 - corr^2) *
    N(0, w_sigma^2) (seed + 1); corr = 0 is the independent second head of the fifth configuration.
    Weights are stored vocabulary-major, [V, hidden]."""
    name: str
    R: int
    V: int
    k: int
    d: int
    g: int
    m: int
    hidden: int
    h_scale: float = 1.0
    w_sigma: float = 0.02
    w_corr: float = 0.0
    ref_sigma: Optional[float] = 0.07
    seed: int = BASE_SEED + 5
    eta: float = 1.0
    eps: float = 0.2
    delta: float = 1e-6
    dtype: str = "bf16"
    full_path: bool = True

    @property
    def rho(self) -> int:
        return 1 + (self.d - 1) * self.k

    @property
    def C(self) -> int:
        return self.k + (self.d - 1) * self.k * self.k

    @property
    def torch_dtype(self):
        return torch.bfloat16


FUSED_CONFIGS: Dict[str, FusedWorkload] = {
    "llama33_70b_fused": FusedWorkload("llama33_70b_fused", R=1024, V=128256, k=8, d=8, g=80, m=8, hidden=8192),
    # the same shape with a target head correlated with the draft head, so that target and draft agree often
    # enough for accepted paths (and hence a backward with real rows) to exist; not one of the five named
    # configurations (whose second head is an independent draw), a companion that exercises the gradient
    "llama33_70b_fused_corr": FusedWorkload("llama33_70b_fused_corr", R=1024, V=128256, k=8, d=8, g=80, m=8,
                                            hidden=8192, w_corr=0.95),
}


def make_fused(w: FusedWorkload, device) -> Dict[str, torch.Tensor]:
    device = torch.device(device)
    s0 = w.seed * 1000003
    s1 = (w.seed + 1) * 1000003
    shape = (w.R, w.d, w.k, w.hidden)
    H_cur = _noise(shape, w.h_scale, device, s0 + 1)
    if w.ref_sigma is None:
        H_ref = _noise(shape, w.h_scale, device, s1 + 1)
    else:
        H_ref = H_cur + _noise(shape, w.ref_sigma, device, s1 + 1)
    out = {"H_cur": H_cur.to(torch.bfloat16), "H_ref": H_ref.to(torch.bfloat16)}
    del H_cur, H_ref
    rows = max(1, (1 << 28) // w.hidden)                      # generate the heads in ~1 GiB fp32 blocks
    W_d = torch.empty((w.V, w.hidden), dtype=torch.bfloat16, device=device)
    W_t = torch.empty((w.V, w.hidden), dtype=torch.bfloat16, device=device)
    c = float(w.w_corr)
    for v0 in range(0, w.V, rows):
        v1 = min(v0 + rows, w.V)
        wd = _noise((v1 - v0, w.hidden), w.w_sigma, device, s0 + 11 + v0)
        wt = _noise((v1 - v0, w.hidden), w.w_sigma, device, s1 + 11 + v0)
        W_d[v0:v1] = wd.to(torch.bfloat16)
        W_t[v0:v1] = (c * wd + math.sqrt(max(0.0, 1.0 - c * c)) * wt).to(torch.bfloat16)
    out["W_draft"] = W_d
    out["W_target"] = W_t
    return out


def algorithmic_bytes(w: Workload, n_models: int = 2) -> int:
    """Bytes the forward path must read: every used draft row and every used
    target row once, for `n_models` trees per root."""
    return 2 * n_models * w.R * w.rho * w.V * w.elem_bytes
