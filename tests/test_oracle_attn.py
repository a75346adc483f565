"""Pins for the oracle's attention (paper Eq. 1; block-sparse form of Sec. 3.2 / Sec. 5.2)
and for Algorithm 1 end to end: explicit-loop dense attention, the keep-all special case,
constant-V and single-block closed forms, log-sum-exp, permutation equivariance, and the
mask cache schedule of Sec. 5.3.
"""
import math

import numpy as np
import pytest

from oracle import dfs_oracle as O
from workloads import CONFIGS, derived_sizes, make_qkv
from workloads.synth import as_f64


def _loop_dense(q, k, v):
    """Eq. 1 as a triple loop."""
    N, d = q.shape
    out = np.zeros((N, v.shape[1]))
    for i in range(N):
        logit = [sum(q[i][c] * k[j][c] for c in range(d)) / math.sqrt(d) for j in range(N)]
        mx = max(logit)
        w = [math.exp(x - mx) for x in logit]
        z = sum(w)
        for j in range(N):
            for c in range(v.shape[1]):
                out[i][c] += w[j] / z * v[j][c]
    return out


def test_dense_attn_is_eq1():
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal((19, 5)) for _ in range(3))
    np.testing.assert_allclose(O.dense_attn(q, k, v), _loop_dense(q, k, v), rtol=1e-12, atol=1e-14)


def test_keep_all_mask_equals_dense_with_ragged_tail():
    rng = np.random.default_rng(1)
    B, N_v, d = 8, 29, 4                        # last block holds 5 real tokens
    M = 4
    q, k, v = (np.zeros((2, M * B, d)) for _ in range(3))
    for x in (q, k, v):
        x[:, :N_v] = rng.standard_normal((2, N_v, d))
    k[:, N_v:] = 50.0                           # pad keys must never be attended to
    v[:, N_v:] = 1e6
    blk_valid = np.array([8, 8, 8, 5])
    o, lse = O.sparse_attn(q, k, v, np.ones((2, M, M), np.uint8), blk_valid, B)
    for h in range(2):
        np.testing.assert_allclose(o[h, :N_v], _loop_dense(q[h, :N_v], k[h, :N_v], v[h, :N_v]), rtol=1e-11, atol=1e-13)
        s = q[h, :N_v] @ k[h, :N_v].T / math.sqrt(d)
        np.testing.assert_allclose(lse[h, :N_v], np.log(np.exp(s).sum(axis=1)), rtol=1e-12)


def test_masked_softmax_is_renormalised_over_kept_blocks():
    rng = np.random.default_rng(2)
    B, M, d = 4, 5, 3
    q, k, v = (rng.standard_normal((1, M * B, d)) for _ in range(3))
    mask = np.zeros((1, M, M), np.uint8)
    keep = {0: [1, 3], 1: [0], 2: [2, 4], 3: [0, 1, 2, 3, 4], 4: [4]}
    for u, cols in keep.items():
        mask[0, u, cols] = 1
    o, _ = O.sparse_attn(q, k, v, mask, np.full(M, B), B)
    for u, cols in keep.items():
        idx = np.concatenate([np.arange(c * B, (c + 1) * B) for c in cols])
        for i in range(u * B, (u + 1) * B):
            logit = np.array([np.dot(q[0, i], k[0, j]) / math.sqrt(d) for j in idx])
            w = np.exp(logit - logit.max()); w /= w.sum()
            np.testing.assert_allclose(o[0, i], sum(wj * v[0, j] for wj, j in zip(w, idx)), rtol=1e-12, atol=1e-14)


def test_constant_value_block_gives_that_constant():
    rng = np.random.default_rng(3)
    B, M, d = 4, 3, 5
    q, k = (rng.standard_normal((1, M * B, d)) for _ in range(2))
    v = np.zeros((1, M * B, d)); v[0, B:2 * B] = 7.5
    mask = np.zeros((1, M, M), np.uint8); mask[0, :, 1] = 1
    o, _ = O.sparse_attn(q, k, v, mask, np.full(M, B), B)
    np.testing.assert_allclose(o, 7.5, rtol=1e-13)


def test_q_blocks_subset_matches_full():
    rng = np.random.default_rng(4)
    B, M, d = 4, 6, 3
    q, k, v = (rng.standard_normal((2, M * B, d)) for _ in range(3))
    mask = (rng.random((2, M, M)) < 0.5).astype(np.uint8); mask[:, np.arange(M), np.arange(M)] = 1
    full, _ = O.sparse_attn(q, k, v, mask, np.full(M, B), B)
    part, _ = O.sparse_attn(q, k, v, mask, np.full(M, B), B, q_blocks=[1, 4])
    np.testing.assert_array_equal(part[:, B:2 * B], full[:, B:2 * B])
    np.testing.assert_array_equal(part[:, 4 * B:5 * B], full[:, 4 * B:5 * B])
    assert np.all(np.isnan(part[:, :B]))


def test_algorithm1_keep_all_equals_dense_on_raster_input():
    """Attention is permutation equivariant: reorder -> dense attention -> inverse reorder
    must reproduce Eq. 1 on the unpermuted tokens (text rows included)."""
    rng = np.random.default_rng(5)
    T, H, W, n_text, B, Bs, d = 3, 4, 5, 6, 16, 4, 4
    N = T * H * W + n_text
    q, k, v = (rng.standard_normal((2, N, d)) for _ in range(3))
    alg = O.DFSAttnOracle(T, H, W, n_text, B, Bs)
    out = alg.step(q, k, v, 0, sparsity=0.0)
    for h in range(2):
        np.testing.assert_allclose(out[h], O.dense_attn(q[h], k[h], v[h]), rtol=1e-10, atol=1e-12)


def test_mask_cache_schedule():
    rng = np.random.default_rng(6)
    T, H, W, B, Bs, d = 2, 4, 8, 8, 4, 4
    N = T * H * W
    alg = O.DFSAttnOracle(T, H, W, 0, B, Bs, delta=3)
    masks = []
    for t in range(7):
        q, k, v = (rng.standard_normal((1, N, d)) * 2 for _ in range(3))
        out = alg.step(q, k, v, t, sparsity=0.5)
        masks.append(alg.mask.copy())
        # outputs are recomputed every step with the step's own Q, K, V under the cached mask
        qp, kp, vp = (O.permute(x, alg.perm_pad) for x in (q, k, v))
        want, _ = O.sparse_attn(qp, kp, vp, alg.mask, alg.blk_valid, B)
        np.testing.assert_array_equal(out, O.unpermute(want, alg.inv))
        if t % 3 == 0:
            fresh, _ = O.select_topk(O.block_score(qp, kp, N, B, Bs), 0.5)
            assert np.array_equal(alg.mask, fresh)
    assert np.array_equal(masks[0], masks[1]) and np.array_equal(masks[1], masks[2])
    assert not np.array_equal(masks[2], masks[3])
    assert np.array_equal(masks[3], masks[5]) and not np.array_equal(masks[5], masks[6])


def test_tiny_workload_generator_and_recall_sanity():
    """The tiny workload end to end on the oracle: kept blocks hold more than their share of
    the true attention mass (recall of Eq. 3 above the budget gamma), and reordering lowers the
    intra-block variance (direction of Table 1).  Qualitative, on synthetic inputs."""
    w = CONFIGS["tiny"]
    sz = derived_sizes(w)
    q, k, v = (as_f64(x) for x in make_qkv(w))
    perm_pad, inv, blk_valid = O.hilbert_perm(w.T, w.H, w.W, 0, w.B)
    qp, kp = O.permute(q, perm_pad), O.permute(k, perm_pad)
    mask, kk = O.select_topk(O.block_score(qp, kp, sz["N_v"], w.B, w.Bs), 0.5)
    assert kk == 2
    for h in range(w.heads):
        s = qp[h] @ kp[h].T / math.sqrt(w.d)
        A = np.exp(s - s.max(axis=1, keepdims=True)); A /= A.sum(axis=1, keepdims=True)
        alpha = A.reshape(sz["M"], w.B, sz["M"], w.B).sum(axis=(1, 3))
        recall = (alpha * mask[h]).sum() / alpha.sum()
        assert recall > 0.5
    var_raster = q[0].reshape(sz["M"], w.B, w.d).var(axis=1).mean()
    var_hilbert = qp[0].reshape(sz["M"], w.B, w.d).var(axis=1).mean()
    assert var_hilbert < var_raster


def test_bf16_rounded_weights_move_the_log_sum_exp_by_their_unit_roundoff():
    """Why the bf16 attention kernel keeps an unrounded sum when the log-sum-exp is asked for.  Its output is
    normalised by the sum of the softmax weights as rounded to bf16 (the weights the matrix product uses).  Taking
    the logarithm of that sum instead of the exact one moves the log-sum-exp by up to bf16's unit roundoff
    2^-8 = 3.9e-3 (8 significant bits, round to nearest), not by 2^-9: reached when one key dominates a row and its
    weight falls halfway between two bf16 values, and approached (3e-3) on ordinary seeded inputs.  Computed here with
    the oracle's logits and plain numpy rounding; nothing of the HIP path is involved."""
    from workloads import Workload
    from workloads.synth import round_to_bf16
    # (a) the worst case by construction: one key, weight 1 + 2^-8 - eps relative to the reference -> rounds to 1
    p = np.array([1.0 + 2.0 ** -8 - 2.0 ** -20], dtype=np.float32)
    err = abs(math.log(float(round_to_bf16(p).astype(np.float64).sum())) - math.log(float(p.astype(np.float64).sum())))
    assert 3.8e-3 < err < 2.0 ** -8
    # (b) seeded inputs, weights relative to the row maximum
    w = Workload("mid_bf16", 5, 12, 20, heads=1, d=128, dtype="bf16", B=128, Bs=32, sparsity=(0.6,), seed=77)
    q, k, v = (as_f64(x) for x in make_qkv(w))
    s = q[0] @ k[0].T / math.sqrt(w.d)
    m = s.max(axis=1, keepdims=True)
    pw = np.exp(s - m)
    exact = np.log(pw.sum(axis=1))
    rounded = np.log(round_to_bf16(pw.astype(np.float32)).astype(np.float64).sum(axis=1))
    worst = np.abs(rounded - exact).max()
    assert 1e-3 < worst <= 2.0 ** -8 * 1.001, worst      # far above any fp32 effect, inside the roundoff bound
