"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/dfsattn.h declares, derives sizes like the oracle does, and turns bad arguments into error
codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

from oracle import dfs_oracle as O
from workloads import CONFIGS, derived_sizes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = pytest.importorskip("paper_2605_23445_amd")


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "dfsattn.h")).read()
    declared = set(re.findall(r"\b(dfs_[a-z_0-9]+)\s*\(", header))
    assert declared == set(P.EXPORTS)
    lib = C.CDLL(P.lib_path())
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("name", list(CONFIGS))
def test_sizes_match_workload_table(name):
    w = CONFIGS[name]
    s = P.dfs_geom_sizes(P.Geom(w.T, w.H, w.W, w.n_text, w.heads, w.d, w.B, w.Bs))
    want = derived_sizes(w)
    got = dict(N_v=s.N_v, N=s.N, M_v=s.M_v, M_x=s.M_x, M=s.M, N_pad=s.N_pad, r=s.r, M_s=s.M_s)
    assert got == want
    assert s.bits == O.cube_bits(w.T, w.H, w.W)
    for sp in w.sparsity:
        assert P.dfs_keep_count(sp, s.M_v) == O.keep_count(sp, s.M_v)


def test_keep_count_matches_oracle_on_a_sweep():
    for M_v in (1, 2, 7, 138, 591, 929, 4096):
        for i in range(0, 101):
            assert P.dfs_keep_count(i / 100, M_v) == O.keep_count(i / 100, M_v)
    assert P.dfs_keep_count(1.5, 10) == 0 and P.dfs_keep_count(0.5, 0) == 0


@pytest.mark.parametrize("bad,code", [
    (dict(d=96), -2), (dict(B=32), -2), (dict(Bs=48), -2), (dict(Bs=8, B=128), -2), (dict(T=0), -2),
    (dict(W=513), -2), (dict(heads=0), -2), (dict(n_text=-1), -2)])
def test_bad_geometry_is_rejected(bad, code):
    base = dict(T=4, H=8, W=8, n_text=0, heads=2, d=64, B=64, Bs=16)
    base.update(bad)
    with pytest.raises(P.DfsError) as e:
        P.dfs_geom_sizes(P.Geom(**base))
    assert e.value.code == code and P.dfs_last_error()
    assert P.dfs_workspace_bytes(P.Geom(**base), P.DFS_WS_FORWARD) == 0


def test_argument_errors_come_before_any_launch():
    """Null pointers, missing workspace and bad enums are refused on the host (no GPU is present here)."""
    lib = C.CDLL(P.lib_path())
    g = P.Geom(4, 8, 8, 0, 2, 64, 64, 16)
    fake = C.c_void_p(0x1000)
    lib.dfs_last_error.restype = C.c_char_p
    vp = C.c_void_p
    lib.dfs_hilbert_perm.argtypes = [C.POINTER(P.Geom), vp, vp, vp, vp, C.c_size_t, vp]
    assert lib.dfs_hilbert_perm(C.byref(g), None, fake, fake, fake, 1 << 20, None) == -1
    assert lib.dfs_hilbert_perm(C.byref(g), fake, fake, fake, None, 0, None) == -4
    assert lib.dfs_hilbert_perm(C.byref(g), fake, fake, fake, C.c_void_p(0x1001), 1 << 20, None) == -4   # misaligned
    assert lib.dfs_hilbert_perm(C.byref(g), fake, fake, fake, fake, 16, None) == -4
    assert b"workspace" in lib.dfs_last_error()
    lib.dfs_permute.argtypes = [C.POINTER(P.Geom), C.c_int, vp, vp, vp, vp]
    assert lib.dfs_permute(C.byref(g), 7, fake, fake, fake, None) == -3
    assert lib.dfs_permute(C.byref(g), 0, fake, None, fake, None) == -1
    lib.dfs_select_mask.argtypes = [C.POINTER(P.Geom), vp, C.c_int, C.c_double, C.c_double, vp, vp, vp, C.c_int32, vp, vp, C.c_size_t, vp]
    assert lib.dfs_select_mask(C.byref(g), fake, 5, 0.5, 0.0, None, fake, fake, 4, None, None, 0, None) == -1
    assert lib.dfs_select_mask(C.byref(g), fake, 0, 1.5, 0.0, None, fake, fake, 4, None, None, 0, None) == -1
    assert lib.dfs_select_mask(C.byref(g), fake, 0, 0.5, 0.0, None, fake, fake, 1, None, None, 0, None) == -2   # K_max below k
    assert lib.dfs_select_mask(C.byref(g), fake, 1, 0.5, 0.9, None, fake, fake, 4, None, None, 0, None) == -4
    lib.dfs_sparse_attn_fwd.argtypes = [C.POINTER(P.Geom), C.c_int, vp, vp, vp, vp, vp, C.c_int32, C.c_float, vp, vp, vp]
    assert lib.dfs_sparse_attn_fwd(C.byref(g), 1, fake, fake, fake, fake, fake, 2, 0.0, fake, None, None) == -1
    assert lib.dfs_sparse_attn_fwd(C.byref(g), 1, fake, fake, None, fake, fake, 2, 0.125, fake, None, None) == -1
    lib.dfs_block_score.argtypes = [C.POINTER(P.Geom), C.c_int, vp, vp, vp, vp, C.c_size_t, vp]
    assert lib.dfs_block_score(C.byref(g), 0, fake, fake, fake, None, 0, None) == -4
    # tensors that do not start on a 16-byte boundary (index arrays: 4-byte) are refused, not read
    odd8, odd2 = C.c_void_p(0x1008), C.c_void_p(0x1002)
    assert lib.dfs_permute(C.byref(g), 0, odd8, fake, fake, None) == -1
    assert b"aligned" in lib.dfs_last_error()
    assert lib.dfs_permute(C.byref(g), 0, fake, odd2, fake, None) == -1
    assert lib.dfs_sparse_attn_fwd(C.byref(g), 1, fake, odd8, fake, fake, fake, 2, 0.125, fake, None, None) == -1
    assert lib.dfs_sparse_attn_fwd(C.byref(g), 1, fake, fake, fake, fake, fake, 2, 0.125, fake, odd2, None) == -1
    assert lib.dfs_block_score(C.byref(g), 0, fake, odd8, fake, fake, 1 << 30, None) == -1


def test_binding_refuses_host_tensors():
    import torch
    g = P.Geom(4, 8, 8, 0, 2, 64, 64, 16)
    x = torch.zeros((2, 256, 64))
    with pytest.raises(ValueError):
        P.dfs_permute(g, P.DFS_F32, x, torch.zeros(256, dtype=torch.int32), x.clone())


def test_schedule_matches_oracle_and_rejects_bad_steps():
    for total in (4, 7, 13, 50, 100):
        for delta in (1, 3, 12):
            for t in range(total):
                for cached in (None, 0.3, 0.2, 0.1):
                    got = P.dfs_schedule(total, t, delta, cached)
                    want = O.paper_schedule(total, t, delta, cached_keep=cached)
                    assert (got[0], got[1], round(got[2], 9)) == (want[0], want[1], round(want[2], 9))
    for bad in ((0, 0, 1), (10, 10, 1), (10, -1, 1), (10, 3, 0)):
        with pytest.raises(P.DfsError):
            P.dfs_schedule(*bad)


def test_build_entry_does_not_need_a_built_library():
    """build() must work in a tree where the library does not exist yet: it may not import the package
    (whose import fails loudly without the library) before it has built it."""
    import ast
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    tree = ast.parse(open(os.path.join(root, "__graft_entry__.py")).read())
    build = next(n for n in tree.body if isinstance(n, ast.FunctionDef) and n.name == "build")
    seen_build_call = False
    for node in ast.walk(build):
        if isinstance(node, ast.Call) and isinstance(node.func, ast.Attribute) and node.func.attr == "build_library":
            seen_build_call = True
    assert seen_build_call
    first_pkg_import = min((n.lineno for n in ast.walk(build)
                            if isinstance(n, (ast.Import, ast.ImportFrom))
                            and any("paper_2605_23445_amd" in (a.name if isinstance(n, ast.Import) else (n.module or "")) for a in n.names)),
                           default=None)
    call_line = next(n.lineno for n in ast.walk(build)
                     if isinstance(n, ast.Call) and isinstance(n.func, ast.Attribute) and n.func.attr == "build_library")
    assert first_pkg_import is None or first_pkg_import > call_line
    # and build.py itself imports nothing from the package
    src = open(os.path.join(root, "paper_2605_23445_amd", "build.py")).read()
    assert "paper_2605_23445_amd" not in src.replace("paper_2605_23445_amd/build.py", "")
