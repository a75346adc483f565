"""dfs_select_mask_static (the entry point that allocates nothing: its scratch is a buffer inside the library)
against dfs_select_mask, through the C ABI: every output bit for bit, on two calls in a row, the second on a
smaller input, so that what the first call left in the shared buffer must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

P = pytest.importorskip("paper_2605_23445_amd")
from tests import gpu_util as G  # noqa: E402


def _scores(heads, M_v, seed):
    rng = np.random.default_rng(seed)
    s = rng.random((heads, M_v, M_v)).astype(np.float32) ** 4
    s[0, 0, :] = 0.25                        # a row of exact ties
    s[heads - 1, M_v - 1, ::2] = 0.0
    return torch.from_numpy(s).cuda()


def _both(g, score, mode, sparsity, mass):
    s = P.dfs_geom_sizes(g)
    K_max = P.dfs_keep_count(sparsity, s.M_v) + s.M_x if mode == P.DFS_SELECT_TOPK else s.M
    ref = G.gpu_select(g, score, mode, sparsity, mass=mass, K_max=K_max)
    mask = torch.full((g.heads, s.M, s.M), 7, dtype=torch.uint8, device="cuda")
    kv_idx = torch.full((g.heads, s.M, K_max), -1, dtype=torch.int32, device="cuda")
    kv_cnt = torch.full((g.heads, s.M), -5, dtype=torch.int32, device="cuda")
    k_head = torch.full((g.heads,), -1, dtype=torch.int32, device="cuda")
    P.dfs_select_mask_static(g, score, mode, sparsity, mass, mask, kv_idx, kv_cnt, K_max, k_head)
    torch.cuda.synchronize()
    assert torch.equal(mask, ref.mask), "mask"
    assert torch.equal(kv_cnt, ref.kv_cnt), "kv_cnt"
    assert torch.equal(kv_idx, ref.kv_idx), "kv_idx"          # both start from -1, so unwritten entries agree too
    assert torch.equal(k_head, ref.k_head), "k_head"


def test_static_scratch_select_equals_workspace_select_twice():
    big = P.Geom(21, 45, 80, 130, 5, 128, 128, 32)            # 591 video + 2 text blocks, 5 heads
    small = P.Geom(3, 9, 11, 0, 2, 64, 64, 16)                # 5 video blocks, 2 heads
    for g, seed in ((big, 1), (small, 2)):
        print(f"static-scratch select: grid {g.T}x{g.H}x{g.W}+{g.n_text}, {g.heads} heads", flush=True)
        score = _scores(g.heads, P.dfs_geom_sizes(g).M_v, seed)
        _both(g, score, P.DFS_SELECT_MASS_HEAD, 0.9, 0.8)
        _both(g, score, P.DFS_SELECT_MASS_ROW, 0.9, 0.8)
        _both(g, score, P.DFS_SELECT_TOPK, 0.75, 0.0)


def test_static_scratch_select_refuses_what_does_not_fit():
    g = P.Geom(64, 128, 128, 0, 64, 64, 128, 32)              # 8192 blocks x 64 heads: 2 MiB of keep counts
    s = P.dfs_geom_sizes(g)
    assert P.dfs_workspace_bytes(g, P.DFS_WS_SELECT_MASK) > (1 << 20)
    one = torch.zeros(1, dtype=torch.float32, device="cuda")
    lib = C.CDLL(P.lib_path())
    lib.dfs_select_mask_static.argtypes = [C.POINTER(P.Geom), C.c_void_p, C.c_int, C.c_double, C.c_double, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.dfs_last_error.restype = C.c_char_p
    p = C.c_void_p(one.data_ptr())                            # never dereferenced: the size check comes first
    rc = lib.dfs_select_mask_static(C.byref(g), p, P.DFS_SELECT_MASS_HEAD, 0.9, 0.8, None, p, p, s.M, None, None)
    assert rc == -4 and b"built-in buffer" in lib.dfs_last_error()
