"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

import paper_2509_22134_amd as G
from paper_2509_22134_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ensure_built():
    if not os.path.exists(G.lib_path()):
        from paper_2509_22134_amd.build import build_lib
        build_lib()


def test_library_exports_every_declared_symbol():
    _ensure_built()
    hdr = open(os.path.join(ROOT, "include", "gto.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(gto_[a-z_0-9]+)\s*\(", hdr))
    assert {"gto_expand_tree", "gto_select_topg", "gto_tree_reward", "gto_group_advantage",
            "gto_ppo_surrogate_fwd", "gto_ppo_surrogate_bwd"} <= names
    lib = C.CDLL(G.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), n
        assert hasattr(G, n), f"python binding lacks {n}"
    assert G.gto_version() >= 100


def test_struct_layout_matches_header():
    assert C.sizeof(B.gto_config) == 80
    assert B.gto_config.row_stride.offset == 24
    assert C.sizeof(B.gto_tree) == 10 * 8 and C.sizeof(B.gto_reward) == 9 * 8


def _cfg(**kw):
    base = dict(R=8, d=3, k=4, g=10, V=1000, dtype=G.GTO_F32, group_size=4)
    base.update(kw)
    return G.make_config(**base)


def _status(fn, *a):
    with pytest.raises(G.GtoError) as e:
        fn(*a)
    return e.value.status


class _Fake:
    """Stands in for a device tensor: validation fails before the pointer is ever used."""
    def __init__(self, ptr=0x1000):
        self._p = ptr

    def data_ptr(self):
        return self._p

    def get(self, *_):
        return self


class _FakeDict(dict):
    def get(self, key, default=None):
        return _Fake()

    def __getitem__(self, key):
        return _Fake()


def test_validation_errors_without_gpu():
    _ensure_built()
    E = {"null": -1, "shape": -2, "align": -3, "dtype": -4, "mode": -5, "ws": -6}
    fake, fd = _Fake(), _FakeDict()
    assert _status(G.gto_draft_row_stats, _cfg(V=3), fake, fd) == E["shape"]          # V < k
    assert _status(G.gto_draft_row_stats, _cfg(k=65, V=100), fake, fd) == E["shape"]
    assert _status(G.gto_draft_row_stats, _cfg(k=20, d=12), fake, fd) == E["shape"]    # C > 4096
    assert _status(G.gto_draft_row_stats, _cfg(g=0), fake, fd) == E["shape"]
    assert _status(G.gto_draft_row_stats, _cfg(d=0), fake, fd) == E["shape"]
    assert _status(G.gto_draft_row_stats, _cfg(R=0), fake, fd) == E["shape"]
    assert _status(G.gto_draft_row_stats, _cfg(row_stride=999), fake, fd) == E["shape"]
    assert _status(G.gto_draft_row_stats, _cfg(V=1001, row_stride=1002), fake, fd) == E["align"]
    assert _status(G.gto_draft_row_stats, _cfg(), _Fake(0x1004), fd) == E["align"]
    assert _status(G.gto_draft_row_stats, _cfg(dtype=7), fake, fd) == E["dtype"]
    assert _status(G.gto_draft_row_stats, _cfg(reward_mode=9), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(eta=0.0), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(), None, fd) == E["null"]
    assert _status(G.gto_draft_row_stats, _cfg(), fake, None) == E["null"]
    assert _status(G.gto_group_advantage, _cfg(group_size=3), fake, fake, fake) == E["shape"]   # R % m != 0
    assert _status(G.gto_group_advantage, _cfg(), None, fake, fake) == E["null"]
    assert _status(G.gto_select_topg, _cfg(), None, fd) == E["null"]
    assert _status(G.gto_tree_reward, _cfg(), fd, None, fd, fd) == E["null"]
    assert _status(G.gto_tree_reward, _cfg(path_mode=3), fd, fake, fd, fd) == E["mode"]
    # the temperature-1 walk needs the caller's uniform numbers
    no_u = {n: fake for n in B._REWARD if n != "accept_u"}
    assert _status(G.gto_tree_reward, _cfg(path_mode=G.GTO_PATH_SAMPLED), fd, fake, fd, no_u) == E["null"]
    # surrogate forward without reference statistics needs a workspace
    assert _status(G.gto_ppo_surrogate_fwd, _cfg(), fd, fd, fake, fd, fake, None, fake, fd) == E["ws"]
    assert "workspace" in G.gto_strerror(E["ws"])
    assert G.gto_workspace_bytes(_cfg()) == 256
    # tuning fields travel in the config and are validated like everything else
    assert _status(G.gto_draft_row_stats, _cfg(waves_per_row=3), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(fused_groups=17), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(fused_groups=9, fused_layout=1), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(fused_layout=2), fake, fd) == E["mode"]
    # NaN / inf / negative parameters are rejected by bit tests (the library is built with NaNs not honoured)
    for bad in (float("nan"), float("inf"), -1.0):
        assert _status(G.gto_draft_row_stats, _cfg(eta=bad), fake, fd) == E["mode"]
        assert _status(G.gto_draft_row_stats, _cfg(eps=bad), fake, fd) == E["mode"]
        assert _status(G.gto_draft_row_stats, _cfg(delta=bad), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(grad_scale=float("nan")), fake, fd) == E["mode"]
    assert _status(G.gto_draft_row_stats, _cfg(eps=0.0, delta=0.0), None, fd) == E["null"]   # zero is allowed


def test_no_process_wide_state_is_exported():
    """Tuning is per call: the library exports no setter and reads no environment variable."""
    _ensure_built()
    lib = C.CDLL(G.lib_path())
    for name in ("gto_set_waves_per_row", "gto_set_fused_tuning"):
        assert not hasattr(lib, name), name
    src = open(os.path.join(ROOT, "paper_2509_22134_amd", "binding.py")).read()
    assert "environ" not in src


def test_library_sources_never_allocate_device_memory():
    """The boundary's ownership rule, checked on the sources: no allocation or free call anywhere."""
    import glob
    for f in glob.glob(os.path.join(ROOT, "paper_2509_22134_amd", "csrc", "*")):
        text = open(f).read()
        for word in ("hipMalloc", "hipFree", "hipHostMalloc", "hipMemset", "hipDeviceSynchronize",
                     "hipStreamSynchronize"):
            assert word not in text, (os.path.basename(f), word)
