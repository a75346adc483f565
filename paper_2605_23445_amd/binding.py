"""ctypes binding of the C ABI in include/dfsattn.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdfsattn.so")

DFS_F32, DFS_BF16 = 0, 1
DFS_SELECT_TOPK, DFS_SELECT_MASS_HEAD, DFS_SELECT_MASS_ROW = 0, 1, 2
DFS_WS_HILBERT_PERM, DFS_WS_BLOCK_SCORE, DFS_WS_SELECT_MASK, DFS_WS_FORWARD, DFS_WS_FORWARD_BF16 = 0, 1, 2, 3, 4


class DfsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"dfsattn error {code}: {msg}")
        self.code = code


class Geom(C.Structure):
    """Mirror of dfs_geom."""
    _fields_ = [(n, C.c_int32) for n in ("T", "H", "W", "n_text", "heads", "d", "B", "Bs")]


class Sizes(C.Structure):
    """Mirror of dfs_sizes."""
    _fields_ = [("N_v", C.c_int64), ("N", C.c_int64), ("N_pad", C.c_int64), ("M_v", C.c_int32), ("M_x", C.c_int32),
                ("M", C.c_int32), ("r", C.c_int32), ("M_s", C.c_int32), ("bits", C.c_int32)]


class _MaskStateC(C.Structure):
    _fields_ = [("kv_idx", C.c_void_p), ("kv_cnt", C.c_void_p), ("mask", C.c_void_p), ("k_head", C.c_void_p),
                ("K_max", C.c_int32)]


@dataclass
class MaskState:
    """Caller-owned mask buffers of one attention layer (kept across diffusion steps)."""
    kv_idx: torch.Tensor
    kv_cnt: torch.Tensor
    mask: torch.Tensor | None
    k_head: torch.Tensor | None
    K_max: int


def lib_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2605_23445_amd/build.py) first - there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, dbl, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_double, C.c_float, C.c_size_t
    gp = C.POINTER(Geom)
    sig = {
        "dfs_geom_sizes": (C.c_int, [gp, C.POINTER(Sizes)]),
        "dfs_workspace_bytes": (sz, [gp, C.c_int]),
        "dfs_last_error": (C.c_char_p, []),
        "dfs_keep_count": (i32, [dbl, i32]),
        "dfs_hilbert_perm": (C.c_int, [gp, vp, vp, vp, vp, sz, vp]),
        "dfs_token_order": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, sz, vp]),
        "dfs_recall": (C.c_int, [gp, vp, vp, vp, vp]),
        "dfs_schedule": (C.c_int, [i32, i32, i32, dbl, C.POINTER(i32), C.POINTER(i32), C.POINTER(dbl)]),
        "dfs_permute": (C.c_int, [gp, C.c_int, vp, vp, vp, vp]),
        "dfs_block_score": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, sz, vp]),
        "dfs_select_mask": (C.c_int, [gp, vp, C.c_int, dbl, dbl, vp, vp, vp, i32, vp, vp, sz, vp]),
        "dfs_select_mask_static": (C.c_int, [gp, vp, C.c_int, dbl, dbl, vp, vp, vp, i32, vp, vp]),
        "dfs_sparse_attn_fwd": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, vp, i32, f32, vp, vp, vp]),
        "dfs_unperm": (C.c_int, [gp, C.c_int, vp, vp, vp, vp]),
        "dfs_block_score_src": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, vp, sz, vp]),
        "dfs_block_score_fused": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, vp, vp, sz, vp]),
        "dfs_sparse_attn_fwd_src": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, vp]),
        "dfs_attn_clock_probe": (C.c_int, [vp]),
        "dfs_probe_mfma": (C.c_int, [i32, i32, vp, vp, vp]),
        "dfs_probe_copy": (C.c_int, [vp, vp, sz, vp]),
        "dfs_probe_read": (C.c_int, [vp, sz, C.c_int32, C.c_int32, vp, vp]),
        "dfs_forward": (C.c_int, [gp, C.c_int, vp, vp, vp, vp, vp, C.c_int, C.c_int, dbl, dbl,
                                  C.POINTER(_MaskStateC), f32, vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()
EXPORTS = ("dfs_geom_sizes", "dfs_workspace_bytes", "dfs_last_error", "dfs_keep_count", "dfs_hilbert_perm", "dfs_permute",
           "dfs_block_score", "dfs_select_mask", "dfs_sparse_attn_fwd", "dfs_unperm", "dfs_forward", "dfs_token_order", "dfs_recall",
           "dfs_schedule", "dfs_block_score_src", "dfs_sparse_attn_fwd_src", "dfs_attn_clock_probe", "dfs_block_score_fused", "dfs_probe_mfma", "dfs_probe_copy", "dfs_probe_read",
           "dfs_select_mask_static")
DFS_ORDER_HILBERT3D, DFS_ORDER_RASTER, DFS_ORDER_HILBERT2D, DFS_ORDER_BLOCK3D = 0, 1, 2, 3


def _check(rc: int):
    if rc != 0:
        raise DfsError(rc, _lib.dfs_last_error().decode())


def _ptr(t: torch.Tensor | None, dtype=None, numel=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL), with shape/dtype checks on the host."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} holds {t.numel()} elements, {numel} needed")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == DFS_BF16 else torch.float32


def dfs_last_error() -> str:
    return _lib.dfs_last_error().decode()


def dfs_geom_sizes(g: Geom) -> Sizes:
    s = Sizes()
    _check(_lib.dfs_geom_sizes(C.byref(g), C.byref(s)))
    return s


def dfs_workspace_bytes(g: Geom, kind: int) -> int:
    return int(_lib.dfs_workspace_bytes(C.byref(g), kind))


def dfs_keep_count(sparsity: float, M_v: int) -> int:
    return int(_lib.dfs_keep_count(float(sparsity), int(M_v)))


def _ws_args(ws: torch.Tensor | None):
    if ws is None:
        return None, 0
    return _ptr(ws, name="ws"), ws.numel() * ws.element_size()


def dfs_hilbert_perm(g: Geom, perm_pad, inv, blk_valid, ws):
    s = dfs_geom_sizes(g)
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_hilbert_perm(C.byref(g), _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"),
                                 _ptr(inv, torch.int32, s.N, "inv"), _ptr(blk_valid, torch.int32, s.M, "blk_valid"),
                                 wp, wb, _stream()))


def dfs_token_order(g: Geom, order: int, perm_pad, inv, blk_valid, ws):
    s = dfs_geom_sizes(g)
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_token_order(C.byref(g), int(order), _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"),
                                _ptr(inv, torch.int32, s.N, "inv"), _ptr(blk_valid, torch.int32, s.M, "blk_valid"),
                                wp, wb, _stream()))


def dfs_recall(g: Geom, lse_sparse, lse_dense, recall):
    s = dfs_geom_sizes(g)
    n = g.heads * s.N_pad
    _check(_lib.dfs_recall(C.byref(g), _ptr(lse_sparse, torch.float32, n, "lse_sparse"), _ptr(lse_dense, torch.float32, n, "lse_dense"),
                           _ptr(recall, torch.float32, g.heads, "recall"), _stream()))


def dfs_schedule(total_steps: int, t: int, delta: int = 12, cached_keep: float | None = None):
    """(dense, refresh, sparsity) of step t under the paper's schedule; cached_keep None = no mask yet."""
    dense, refresh, sparsity = C.c_int32(), C.c_int32(), C.c_double()
    _check(_lib.dfs_schedule(int(total_steps), int(t), int(delta), -1.0 if cached_keep is None else float(cached_keep),
                             C.byref(dense), C.byref(refresh), C.byref(sparsity)))
    return bool(dense.value), bool(refresh.value), sparsity.value


def dfs_permute(g: Geom, dtype: int, x, perm_pad, x_perm):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    _check(_lib.dfs_permute(C.byref(g), dtype, _ptr(x, td, g.heads * s.N * g.d, "x"),
                            _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"),
                            _ptr(x_perm, td, g.heads * s.N_pad * g.d, "x_perm"), _stream()))


def dfs_block_score(g: Geom, dtype: int, q_perm, k_perm, score, ws):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    n = g.heads * s.N_pad * g.d
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_block_score(C.byref(g), dtype, _ptr(q_perm, td, n, "q_perm"), _ptr(k_perm, td, n, "k_perm"),
                                _ptr(score, torch.float32, g.heads * s.M_v * s.M_v, "score"), wp, wb, _stream()))


def dfs_select_mask(g: Geom, score, mode: int, sparsity: float, mass: float, mask, kv_idx, kv_cnt, K_max: int,
                    k_head, ws):
    s = dfs_geom_sizes(g)
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_select_mask(C.byref(g), _ptr(score, torch.float32, g.heads * s.M_v * s.M_v, "score"), mode,
                                float(sparsity), float(mass), _ptr(mask, torch.uint8, g.heads * s.M * s.M, "mask"),
                                _ptr(kv_idx, torch.int32, g.heads * s.M * K_max, "kv_idx"),
                                _ptr(kv_cnt, torch.int32, g.heads * s.M, "kv_cnt"), int(K_max),
                                _ptr(k_head, torch.int32, g.heads, "k_head"), wp, wb, _stream()))


def dfs_select_mask_static(g: Geom, score, mode: int, sparsity: float, mass: float, mask, kv_idx, kv_cnt, K_max: int, k_head):
    s = dfs_geom_sizes(g)
    _check(_lib.dfs_select_mask_static(C.byref(g), _ptr(score, torch.float32, g.heads * s.M_v * s.M_v, "score"), mode,
                                       float(sparsity), float(mass), _ptr(mask, torch.uint8, g.heads * s.M * s.M, "mask"),
                                       _ptr(kv_idx, torch.int32, g.heads * s.M * K_max, "kv_idx"),
                                       _ptr(kv_cnt, torch.int32, g.heads * s.M, "kv_cnt"), int(K_max),
                                       _ptr(k_head, torch.int32, g.heads, "k_head"), _stream()))


def dfs_sparse_attn_fwd(g: Geom, dtype: int, q_perm, k_perm, v_perm, kv_idx, kv_cnt, K_max: int, scale: float,
                        o_perm, lse=None):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    n = g.heads * s.N_pad * g.d
    _check(_lib.dfs_sparse_attn_fwd(C.byref(g), dtype, _ptr(q_perm, td, n, "q_perm"), _ptr(k_perm, td, n, "k_perm"),
                                    _ptr(v_perm, td, n, "v_perm"),
                                    _ptr(kv_idx, torch.int32, g.heads * s.M * K_max, "kv_idx"),
                                    _ptr(kv_cnt, torch.int32, g.heads * s.M, "kv_cnt"), int(K_max), float(scale),
                                    _ptr(o_perm, td, n, "o_perm"), _ptr(lse, torch.float32, g.heads * s.N_pad, "lse"),
                                    _stream()))


def dfs_block_score_src(g: Geom, dtype: int, q, perm_pad, k_perm, score, ws):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_block_score_src(C.byref(g), dtype, _ptr(q, td, g.heads * s.N * g.d, "q"),
                                    _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"),
                                    _ptr(k_perm, td, g.heads * s.N_pad * g.d, "k_perm"),
                                    _ptr(score, torch.float32, g.heads * s.M_v * s.M_v, "score"), wp, wb, _stream()))


def dfs_block_score_fused(g: Geom, dtype: int, q, k, perm_pad, k_perm, score, ws):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_block_score_fused(C.byref(g), dtype, _ptr(q, td, g.heads * s.N * g.d, "q"), _ptr(k, td, g.heads * s.N * g.d, "k"),
                                      _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"),
                                      _ptr(k_perm, td, g.heads * s.N_pad * g.d, "k_perm"),
                                      _ptr(score, torch.float32, g.heads * s.M_v * s.M_v, "score"), wp, wb, _stream()))


def dfs_sparse_attn_fwd_src(g: Geom, dtype: int, q, perm_pad, k_perm, v_perm, kv_idx, kv_cnt, K_max: int, scale: float, o,
                            lse=None):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    n_src, n_perm = g.heads * s.N * g.d, g.heads * s.N_pad * g.d
    _check(_lib.dfs_sparse_attn_fwd_src(C.byref(g), dtype, _ptr(q, td, n_src, "q"), _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"),
                                        _ptr(k_perm, td, n_perm, "k_perm"), _ptr(v_perm, td, n_perm, "v_perm"),
                                        _ptr(kv_idx, torch.int32, g.heads * s.M * K_max, "kv_idx"),
                                        _ptr(kv_cnt, torch.int32, g.heads * s.M, "kv_cnt"), int(K_max), float(scale),
                                        _ptr(o, td, n_src, "o"), _ptr(lse, torch.float32, g.heads * s.N_pad, "lse"), _stream()))


def dfs_attn_clock_probe(counters: torch.Tensor | None):
    """Diagnostic: accumulate shader-clock cycles / 100 MHz ticks / work-group count of the bf16 attention
    kernel into `counters` (3 x int64 on the device, zeroed by the caller); None switches it off."""
    _check(_lib.dfs_attn_clock_probe(_ptr(counters, torch.int64, 3, "counters")))


def dfs_probe_mfma(work_groups: int, iters: int, sink: torch.Tensor, counters: torch.Tensor | None = None):
    """Measurement probe: bare matrix-instruction chains (work_groups x 4 waves x iters x 4 instructions)."""
    _check(_lib.dfs_probe_mfma(int(work_groups), int(iters), _ptr(sink, torch.float32, work_groups * 256, "sink"),
                               _ptr(counters, torch.int64, 2, "counters"), _stream()))


def dfs_probe_copy(src: torch.Tensor, dst: torch.Tensor):
    """Measurement probe: plain device copy, 16 bytes per lane."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(_lib.dfs_probe_copy(_ptr(src), _ptr(dst), n, _stream()))


def dfs_probe_read(src: torch.Tensor, work_groups: int, pieces_per_wg: int, sink: torch.Tensor):
    """Measurement probe: read-only traffic, random 64 KB pieces of `src` (size a multiple of 64 KB)."""
    n = src.numel() * src.element_size()
    _check(_lib.dfs_probe_read(_ptr(src), n, int(work_groups), int(pieces_per_wg), _ptr(sink, torch.int32, 1, "sink"), _stream()))


def dfs_unperm(g: Geom, dtype: int, o_perm, inv, o):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    _check(_lib.dfs_unperm(C.byref(g), dtype, _ptr(o_perm, td, g.heads * s.N_pad * g.d, "o_perm"),
                           _ptr(inv, torch.int32, s.N, "inv"), _ptr(o, td, g.heads * s.N * g.d, "o"), _stream()))


def dfs_forward(g: Geom, dtype: int, q, k, v, perm_pad, inv, refresh: bool, mode: int, sparsity: float, mass: float,
                st: MaskState, scale: float, o, ws):
    s = dfs_geom_sizes(g)
    td = _torch_dtype(dtype)
    n = g.heads * s.N * g.d
    cst = _MaskStateC(_ptr(st.kv_idx, torch.int32, g.heads * s.M * st.K_max, "kv_idx"),
                      _ptr(st.kv_cnt, torch.int32, g.heads * s.M, "kv_cnt"),
                      _ptr(st.mask, torch.uint8, g.heads * s.M * s.M, "mask"),
                      _ptr(st.k_head, torch.int32, g.heads, "k_head"), int(st.K_max))
    wp, wb = _ws_args(ws)
    _check(_lib.dfs_forward(C.byref(g), dtype, _ptr(q, td, n, "q"), _ptr(k, td, n, "k"), _ptr(v, td, n, "v"),
                            _ptr(perm_pad, torch.int32, s.N_pad, "perm_pad"), _ptr(inv, torch.int32, s.N, "inv"),
                            int(bool(refresh)), mode, float(sparsity), float(mass), C.byref(cst), float(scale),
                            _ptr(o, td, n, "o"), wp, wb, _stream()))
