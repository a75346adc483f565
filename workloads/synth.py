"""Seeded Q/K/V generator with the value structure of video-DiT activations.

The paper measures on real activations of HunyuanVideo and Wan2.1; those weights
are not available here, so inputs are synthetic.  Their structure follows the
paper's token model (Assumption 4.1: a smooth component shared by neighbouring
tokens plus independent token noise) and its observation that semantic relevance
follows spatio-temporal proximity (Sec. 5.1):

  field_h(p)[c] = sqrt(2/F) * sum_f a[f,c] * cos(omega_f . p + phi[f,c]),  p = (t,h,w)
  Q = field + sigma*eps_q + u            K = field + sigma*eps_k (+ 4*sqrt(d)*u on sinks)
  V ~ N(0,1)                             (or field + sigma*eps_v for the tiny case)

with F = 8 random frequencies omega_f ~ N(0, I/ell^2) per head, a few high-norm
"sink" key tokens per frame, and optional appended text rows ~ N(0,1).  Everything
is drawn on the host with numpy PCG64 streams keyed by
(seed, tensor id, head), so any head can be generated on its own.

Nothing here computes any step of the attention method.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import Workload

_F = 8


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return ((b + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the fp32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array rounded to the nearest bf16 value, returned as fp32."""
    return bf16_bits_to_f32(to_bf16_bits(x))


def _positions(w: Workload) -> np.ndarray:
    t, h, x = np.meshgrid(np.arange(w.T), np.arange(w.H), np.arange(w.W), indexing="ij")
    return np.stack([t.ravel(), h.ravel(), x.ravel()], axis=1).astype(np.float64)  # raster order


def _field(w: Workload, head: int, pos: np.ndarray) -> np.ndarray:
    rng = np.random.default_rng([w.seed, 0, head])
    omega = rng.standard_normal((_F, 3)) / w.ell
    a = rng.standard_normal((_F, w.d))
    phi = rng.uniform(0.0, 2.0 * np.pi, (_F, w.d))
    ang = pos @ omega.T                                    # [N_v, F]
    # cos(x + phi) = cos x cos phi - sin x sin phi, so the field is two thin products
    f = np.cos(ang) @ (a * np.cos(phi)) - np.sin(ang) @ (a * np.sin(phi))
    return (np.sqrt(2.0 / _F) * f).astype(np.float32)


def sink_tokens(w: Workload) -> np.ndarray:
    """Raster indices of the high-norm key tokens (the same for every head)."""
    if w.sinks_per_frame <= 0:
        return np.zeros(0, dtype=np.int64)
    rng = np.random.default_rng([w.seed, 4])
    out = []
    for t in range(w.T):
        cells = rng.choice(w.H * w.W, size=w.sinks_per_frame, replace=False)
        out.append(t * w.H * w.W + np.sort(cells))
    return np.concatenate(out).astype(np.int64)


def make_head(w: Workload, head: int, pos: np.ndarray | None = None):
    """Q, K, V of one head as fp32 arrays [N, d] in raster order (text rows last)."""
    if pos is None:
        pos = _positions(w)
    N_v = pos.shape[0]
    field = _field(w, head, pos)
    eq = np.random.default_rng([w.seed, 1, head]).standard_normal((N_v, w.d), dtype=np.float32)
    ek = np.random.default_rng([w.seed, 2, head]).standard_normal((N_v, w.d), dtype=np.float32)
    ev = np.random.default_rng([w.seed, 3, head]).standard_normal((N_v, w.d), dtype=np.float32)
    q = field + np.float32(w.sigma) * eq
    k = field + np.float32(w.sigma) * ek
    v = field + np.float32(w.sigma) * ev if w.v_from_field else ev
    sinks = sink_tokens(w)
    if sinks.size:
        u = np.random.default_rng([w.seed, 5, head]).standard_normal(w.d)
        u = (u / np.linalg.norm(u)).astype(np.float32)
        q = q + u
        k[sinks] += np.float32(4.0 * np.sqrt(w.d)) * u
    if w.n_text:
        tx = np.random.default_rng([w.seed, 6, head]).standard_normal((3, w.n_text, w.d), dtype=np.float32)
        q = np.concatenate([q, tx[0]], axis=0)
        k = np.concatenate([k, tx[1]], axis=0)
        v = np.concatenate([v, tx[2]], axis=0)
    return q.astype(np.float32), k.astype(np.float32), v.astype(np.float32)


def make_qkv(w: Workload, heads=None, threads: int = 0):
    """Q, K, V as [heads, N, d] arrays in raster order.

    For a bf16 workload the arrays hold bf16 bit patterns (uint16); for an f32
    workload they hold float32.  `heads` may be an iterable of head indices to
    generate a subset (each head's stream is independent of the others).
    """
    head_ids = list(range(w.heads)) if heads is None else list(heads)
    pos = _positions(w)
    N = pos.shape[0] + w.n_text
    dt = np.uint16 if w.dtype == "bf16" else np.float32
    q = np.empty((len(head_ids), N, w.d), dtype=dt)
    k = np.empty_like(q)
    v = np.empty_like(q)

    def one(i):
        qh, kh, vh = make_head(w, head_ids[i], pos)
        if w.dtype == "bf16":
            q[i], k[i], v[i] = to_bf16_bits(qh), to_bf16_bits(kh), to_bf16_bits(vh)
        else:
            q[i], k[i], v[i] = qh, kh, vh

    workers = min(len(head_ids), threads if threads else min(16, os.cpu_count() or 1))
    if workers > 1:      # heads are independent streams; numpy releases the GIL in its kernels
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(one, range(len(head_ids))))
    else:
        for i in range(len(head_ids)):
            one(i)
    return q, k, v


def as_f64(x: np.ndarray) -> np.ndarray:
    """Exact up-conversion of a generated array (bf16 bits or fp32) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)
