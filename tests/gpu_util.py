"""Helpers for the GPU parity tests: run the stages of the HIP path through the C-ABI binding and
hand results back as numpy arrays.  No arithmetic of the method lives here."""
from __future__ import annotations

import math

import numpy as np
import torch

import paper_2605_23445_amd as P
from workloads import Workload, derived_sizes


def geom_of(w: Workload, heads=None) -> P.Geom:
    return P.Geom(w.T, w.H, w.W, w.n_text, w.heads if heads is None else heads, w.d, w.B, w.Bs)


def dtype_of(w: Workload) -> int:
    return P.DFS_BF16 if w.dtype == "bf16" else P.DFS_F32


def to_dev(x: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(x)
    if x.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).cpu().numpy()
    return t.cpu().numpy()


def ws_tensor(nbytes: int) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


def gpu_perm(g: P.Geom):
    s = P.dfs_geom_sizes(g)
    perm_pad = torch.full((s.N_pad,), -7, dtype=torch.int32, device="cuda")
    inv = torch.full((s.N,), -7, dtype=torch.int32, device="cuda")
    blk_valid = torch.full((s.M,), -7, dtype=torch.int32, device="cuda")
    ws = ws_tensor(P.dfs_workspace_bytes(g, P.DFS_WS_HILBERT_PERM))
    P.dfs_hilbert_perm(g, perm_pad, inv, blk_valid, ws)
    return perm_pad, inv, blk_valid


def gpu_permute(g, dtype, x, perm_pad):
    s = P.dfs_geom_sizes(g)
    out = torch.empty((g.heads, s.N_pad, g.d), dtype=x.dtype, device="cuda")
    P.dfs_permute(g, dtype, x, perm_pad, out)
    return out


def gpu_score(g, dtype, qp, kp):
    s = P.dfs_geom_sizes(g)
    score = torch.full((g.heads, s.M_v, s.M_v), float("nan"), dtype=torch.float32, device="cuda")
    ws = ws_tensor(P.dfs_workspace_bytes(g, P.DFS_WS_BLOCK_SCORE))
    P.dfs_block_score(g, dtype, qp, kp, score, ws)
    return score


def gpu_select(g, score, mode, sparsity, mass=0.0, K_max=None, want_mask=True):
    s = P.dfs_geom_sizes(g)
    if K_max is None:
        K_max = P.dfs_keep_count(sparsity, s.M_v) + s.M_x if mode == P.DFS_SELECT_TOPK else s.M
    mask = torch.full((g.heads, s.M, s.M), 9, dtype=torch.uint8, device="cuda") if want_mask else None
    kv_idx = torch.full((g.heads, s.M, K_max), -1, dtype=torch.int32, device="cuda")
    kv_cnt = torch.full((g.heads, s.M), -1, dtype=torch.int32, device="cuda")
    k_head = torch.full((g.heads,), -1, dtype=torch.int32, device="cuda")
    ws = ws_tensor(P.dfs_workspace_bytes(g, P.DFS_WS_SELECT_MASK))
    P.dfs_select_mask(g, score, mode, sparsity, mass, mask, kv_idx, kv_cnt, K_max, k_head, ws)
    return P.MaskState(kv_idx, kv_cnt, mask, k_head, K_max)


def lists_of_mask(mask_np: np.ndarray, K_max: int):
    """(kv_idx, kv_cnt) in the library's list format for a 0/1 mask [heads, M, M]: ascending kept columns, -1
    beyond the count.  The library's convention, not the method's: a row that keeps all M blocks carries no
    list (kv_cnt == M means dense), so K_max need not hold it."""
    heads, M, _ = mask_np.shape
    kv_idx = np.full((heads, M, K_max), -1, dtype=np.int32)
    kv_cnt = mask_np.sum(axis=2).astype(np.int32)
    for h in range(heads):
        for u in range(M):
            if kv_cnt[h, u] < M or M <= K_max:
                cols = np.nonzero(mask_np[h, u])[0]
                kv_idx[h, u, :cols.size] = cols
    return kv_idx, kv_cnt


def upload_mask(mask_np: np.ndarray, K_max=None) -> P.MaskState:
    """Device kv lists built on the host from a 0/1 mask [heads, M, M] (rows that keep all M blocks get
    no list, like the library's own)."""
    heads, M, _ = mask_np.shape
    cnt = mask_np.sum(axis=2).astype(np.int32)
    if K_max is None:
        K_max = max(1, int(cnt[cnt < M].max()) if np.any(cnt < M) else 1)
    idx = np.full((heads, M, K_max), -1, dtype=np.int32)
    for h in range(heads):
        for u in range(M):
            if cnt[h, u] < M:
                cols = np.nonzero(mask_np[h, u])[0]
                idx[h, u, :cols.size] = cols
    return P.MaskState(torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(), None, None, K_max)


def gpu_attn(g, dtype, qp, kp, vp, st: P.MaskState, want_lse=True, scale=None):
    s = P.dfs_geom_sizes(g)
    o = torch.empty_like(qp)
    lse = torch.full((g.heads, s.N_pad), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    P.dfs_sparse_attn_fwd(g, dtype, qp, kp, vp, st.kv_idx, st.kv_cnt, st.K_max,
                          1.0 / math.sqrt(g.d) if scale is None else scale, o, lse)
    return o, lse


def gpu_unperm(g, dtype, op, inv):
    s = P.dfs_geom_sizes(g)
    o = torch.empty((g.heads, s.N, g.d), dtype=op.dtype, device="cuda")
    P.dfs_unperm(g, dtype, op, inv, o)
    return o


def as_f64_dev(t: torch.Tensor) -> np.ndarray:
    """Exact up-conversion of a device tensor (bf16 or fp32) to a float64 numpy array."""
    return t.to(torch.float32).cpu().numpy().astype(np.float64)
