"""Workload table: the shapes the attention path is tested and timed on.

The five entries follow the shapes of the video DiTs the paper evaluates
(HunyuanVideo 129 frames 720p, Wan2.1 81 frames 720p; Sec. 6.1) plus a
CogVideoX-shaped and a tiny case.  Block size 128 is the paper's (Sec. 6.1);
sub-block sizes 16/32 are two of the sizes of its Table 4.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    H: int
    W: int
    heads: int
    d: int
    dtype: str            # "f32" or "bf16"
    B: int                # block size
    Bs: int               # sub-block size
    sparsity: Tuple[float, ...]
    n_text: int = 0       # appended tokens that are always kept dense
    seed: int = 1000
    ell: float = 3.0      # locality length scale of the positional field, in tokens
    sigma: float = 0.5    # token noise on Q and K
    sinks_per_frame: int = 4
    v_from_field: bool = False
    # mask-caching schedule (only the last workload uses it)
    steps: int = 1
    delta: int = 1
    drift: float = 0.0
    mass: float = 0.0     # >0: adaptive per-head ratio by cumulative score mass
    cap: float = 0.95     # sparsity cap of the adaptive mode

    def with_heads(self, heads: int) -> "Workload":
        return replace(self, heads=heads)


def derived_sizes(w: Workload) -> dict:
    """Token and block counts that follow from a workload's geometry."""
    N_v = w.T * w.H * w.W
    M_v = -(-N_v // w.B)
    M_x = -(-w.n_text // w.B)
    M = M_v + M_x
    r = w.B // w.Bs
    return dict(N_v=N_v, N=N_v + w.n_text, M_v=M_v, M_x=M_x, M=M, N_pad=M * w.B,
                r=r, M_s=M_v * r)


CONFIGS = {
    "tiny": Workload("tiny", 4, 8, 8, heads=2, d=64, dtype="f32", B=64, Bs=16,
                     sparsity=(0.5,), seed=1001, ell=2.0, sigma=0.3,
                     sinks_per_frame=0, v_from_field=True),
    "cogvideox": Workload("cogvideox", 13, 30, 45, heads=48, d=64, dtype="bf16",
                          B=128, Bs=32, sparsity=(0.85,), seed=1002),
    "wan": Workload("wan", 21, 45, 80, heads=40, d=128, dtype="bf16",
                    B=128, Bs=32, sparsity=(0.8, 0.9, 0.95), seed=1003),
    "hunyuan": Workload("hunyuan", 33, 45, 80, heads=24, d=128, dtype="bf16",
                        B=128, Bs=32, sparsity=(0.9,), n_text=256, seed=1004),
    "wan_cache": Workload("wan_cache", 21, 45, 80, heads=40, d=128, dtype="bf16",
                          B=128, Bs=32, sparsity=(0.95,), seed=1005,
                          steps=50, delta=5, drift=0.02, mass=0.9, cap=0.95),
}
