"""Pins for the oracle's hierarchical block score (paper Sec. 5.2, Eq. 2, Eq. 8) and its
selection rules (Eq. 9).  Each pin is independent of the oracle's own formulas: explicit
loops over the definitions, a closed form that ties the score to the true block mass of
Eq. 6, the centroid special case of Defs. 4.2-4.3, counting brute force for the ranking.
"""
import math

import numpy as np
import pytest

from oracle import dfs_oracle as O


def _brute_block_score(qp, kp, N_v, B, Bs):
    """Eq. 2 and Eq. 8 with explicit loops: centroids, every sub-block logit, softmax, sums."""
    N_pad, d = qp.shape
    M_v = -(-N_v // B)
    r = B // Bs
    M_s = M_v * r

    def centroid(x, s):
        rows = [p for p in range(s * Bs, (s + 1) * Bs) if p < N_v]
        if not rows:
            return None
        return [sum(x[p][c] for p in rows) / len(rows) for c in range(d)]

    qc = [centroid(qp, s) for s in range(M_s)]
    kc = [centroid(kp, s) for s in range(M_s)]
    S = [[0.0] * M_v for _ in range(M_v)]
    for i in range(M_s):
        if qc[i] is None:
            continue
        logit = {j: sum(a * b for a, b in zip(qc[i], kc[j])) / math.sqrt(d) for j in range(M_s) if kc[j] is not None}
        mx = max(logit.values())
        z = sum(math.exp(v - mx) for v in logit.values())
        for j, v in logit.items():
            S[i // r][j // r] += math.exp(v - mx) / z
    return np.array(S)


@pytest.mark.parametrize("N_v,B,Bs", [(64, 16, 4), (50, 16, 8), (37, 8, 2), (33, 16, 16)])
def test_block_score_brute_force(N_v, B, Bs):
    rng = np.random.default_rng(N_v)
    d = 6
    N_pad = -(-N_v // B) * B
    qp = np.zeros((2, N_pad, d))
    kp = np.zeros((2, N_pad, d))
    qp[:, :N_v] = rng.standard_normal((2, N_v, d)) * 1.5
    kp[:, :N_v] = rng.standard_normal((2, N_v, d)) * 1.5
    got = O.block_score(qp, kp, N_v, B, Bs)
    for h in range(2):
        np.testing.assert_allclose(got[h], _brute_block_score(qp[h], kp[h], N_v, B, Bs), rtol=1e-12, atol=1e-14)


def test_row_sums_count_live_query_subblocks():
    rng = np.random.default_rng(1)
    N_v, B, Bs, d = 70, 32, 8, 5        # last block: sub-blocks with 6, 0, 0, 0 real tokens... (70-64)
    N_pad = 96
    qp = np.zeros((1, N_pad, d)); kp = np.zeros((1, N_pad, d))
    qp[:, :N_v] = rng.standard_normal((1, N_v, d)); kp[:, :N_v] = rng.standard_normal((1, N_v, d))
    S = O.block_score(qp, kp, N_v, B, Bs)[0]
    np.testing.assert_allclose(S.sum(axis=1), [4, 4, 1], rtol=1e-12)
    # empty key sub-blocks carry no probability: column 2 only holds the one live sub-block
    assert np.all(S >= 0)


def test_closed_form_against_true_block_mass():
    """If Q and K are constant inside every sub-block then A_ij = A_hat_{i'j'} / B_s, so the
    true block mass of Eq. 6 is alpha_uv = B_s * S_hat_uv (from Eq. 1 and Eq. 8)."""
    rng = np.random.default_rng(2)
    B, Bs, M_v, d = 16, 4, 5, 7
    N = B * M_v
    qs = rng.standard_normal((N // Bs, d)) * 1.3
    ks = rng.standard_normal((N // Bs, d)) * 1.3
    q = np.repeat(qs, Bs, axis=0); k = np.repeat(ks, Bs, axis=0)
    # Eq. 1 written out with loops
    A = np.zeros((N, N))
    for i in range(N):
        row = [math.exp(float(np.dot(q[i], k[j])) / math.sqrt(d)) for j in range(N)]
        z = sum(row)
        A[i] = [x / z for x in row]
    alpha = A.reshape(M_v, B, M_v, B).sum(axis=(1, 3))
    S = O.block_score(q[None], k[None], N, B, Bs)[0]
    np.testing.assert_allclose(alpha, Bs * S, rtol=1e-11)


def test_without_subblocks_ranking_is_centroid_dot_product():
    """B_s = B (Table 4 'w/o sub-block'): within a row the softmax is monotone in the logit,
    so ranking S_hat equals ranking <q_hat_u, k_hat_v> (Defs. 4.2-4.3)."""
    rng = np.random.default_rng(3)
    B, M_v, d = 8, 9, 5
    q = rng.standard_normal((1, B * M_v, d)); k = rng.standard_normal((1, B * M_v, d))
    S = O.block_score(q, k, B * M_v, B, B)[0]
    qc = q[0].reshape(M_v, B, d).mean(axis=1); kc = k[0].reshape(M_v, B, d).mean(axis=1)
    dots = qc @ kc.T
    for u in range(M_v):
        assert np.array_equal(np.argsort(-S[u], kind="stable"), np.argsort(-dots[u], kind="stable"))
    mask, kk = O.select_topk(S[None], 0.6)
    assert kk == 4
    for u in range(M_v):
        assert set(np.nonzero(mask[0, u])[0]) == set(np.argsort(-dots[u])[:4])


# ------------------------------------------------------------------ selection (Eq. 9)

def test_keep_count_at_workload_shapes():
    f = np.float32
    assert O.keep_count(0.5, 4) == 2
    assert O.keep_count(float(f(0.85)), 138) == 21
    assert [O.keep_count(float(f(s)), 591) for s in (0.8, 0.9, 0.95)] == [119, 60, 30]
    assert O.keep_count(0.9, 929) == 93
    assert O.keep_count(0.75, 8) == 2          # exact product is not rounded up
    assert O.keep_count(1.0, 10) == 1 and O.keep_count(0.0, 10) == 10


def _brute_topk_row(row, k):
    """Column j is kept iff fewer than k columns beat it (higher score, or equal and lower index)."""
    keep = []
    for j in range(len(row)):
        beat = sum(1 for i in range(len(row)) if row[i] > row[j] or (row[i] == row[j] and i < j))
        if beat < k:
            keep.append(j)
    return keep


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_topk_counting_brute_force(seed):
    rng = np.random.default_rng(seed)
    M_v = 23
    score = rng.random((2, M_v, M_v)).astype(np.float32)
    score[0, 3, :] = 0.25                       # a row of exact ties
    score[1, 5, ::2] = score[1, 5, 1]           # many duplicates of one value
    score = np.round(score * 8) / 8 if seed == 2 else score   # coarse grid: ties everywhere
    mask, k = O.select_topk(score, 0.7)
    assert k == 7
    for h in range(2):
        for u in range(M_v):
            assert list(np.nonzero(mask[h, u])[0]) == _brute_topk_row(score[h, u], k)
    assert np.all(mask.sum(axis=2) == k)


def test_select_tie_break_by_hand():
    score = np.array([[[1.0, 3.0, 3.0, 2.0, 3.0],
                       [0.0, 0.0, 0.0, 0.0, 0.0],
                       [5.0, 4.0, 3.0, 2.0, 1.0],
                       [1.0, 2.0, 3.0, 4.0, 5.0],
                       [2.0, 2.0, 9.0, 2.0, 2.0]]], dtype=np.float32)
    mask, k = O.select_topk(score, 0.6)         # keep 2 of 5
    assert k == 2
    assert [list(np.nonzero(r)[0]) for r in mask[0]] == [[1, 2], [0, 1], [0, 1], [3, 4], [0, 2]]


def test_text_blocks_stay_dense():
    rng = np.random.default_rng(4)
    score = rng.random((1, 6, 6)).astype(np.float32)
    mask, k = O.select_topk(score, 0.5, M_x=2)
    assert mask.shape == (1, 8, 8)
    assert np.all(mask[0, :6, 6:] == 1) and np.all(mask[0, 6:, :] == 1)
    assert np.all(mask[0, :6, :6].sum(axis=1) == k)
    kv_idx, kv_cnt = O.mask_to_lists(mask, 8)
    assert np.all(kv_cnt[0, :6] == k + 2) and np.all(kv_cnt[0, 6:] == 8)
    for u in range(8):
        cols = kv_idx[0, u, :kv_cnt[0, u]]
        assert np.all(np.diff(cols) > 0) and np.all(mask[0, u, cols] == 1)


def test_mass_rule_closed_forms():
    M_v = 40
    uniform = np.full(M_v, 0.1, dtype=np.float32)
    assert O.mass_keep_count(uniform, 0.9) == math.ceil(0.9 * M_v)
    onehot = np.zeros(M_v, dtype=np.float32); onehot[17] = 4.0
    assert O.mass_keep_count(onehot, 0.9) == 1
    assert O.mass_keep_count(np.zeros(M_v, dtype=np.float32), 0.9) == 1
    # geometric row 1/2, 1/4, ...: top-k holds 1 - 2^-k of (1 - 2^-40); 0.9 needs k = 4
    geo = (0.5 ** np.arange(1, M_v + 1)).astype(np.float32)
    assert O.mass_keep_count(geo[::-1].copy(), 0.9) == 4
    # per head: one-hot rows everywhere -> floor at the cap's keep count
    score = np.zeros((1, M_v, M_v), dtype=np.float32)
    score[0, np.arange(M_v), (np.arange(M_v) * 7) % M_v] = 1.0
    mask, k_head = O.select_mass_head(score, 0.9, 0.95)
    assert k_head[0] == O.keep_count(0.95, M_v) == 2
    assert np.all(mask[0].sum(axis=1) == 2)
    assert all(mask[0, u, (u * 7) % M_v] == 1 for u in range(M_v))
    # uniform rows -> every head keeps ceil(mass * M_v)
    mask, k_head = O.select_mass_head(np.full((2, M_v, M_v), 0.025, dtype=np.float32), 0.9, 0.95)
    assert list(k_head) == [36, 36] and np.all(mask.sum(axis=2) == 36)


def test_mass_rule_brute_force_mean():
    rng = np.random.default_rng(5)
    M_v = 31
    score = (rng.random((3, M_v, M_v)) ** 6).astype(np.float32)
    mask, k_head = O.select_mass_head(score, 0.8, 0.9)
    for h in range(3):
        ks = []
        for u in range(M_v):
            row = np.sort(score[h, u].astype(np.float64))[::-1]
            c = np.cumsum(row)
            ks.append(int(np.searchsorted(c, 0.8 * c[-1] * (1 - 1e-9)) + 1))   # float version, away from ties
        want = max(math.ceil(sum(ks) / M_v), O.keep_count(0.9, M_v))
        assert abs(int(k_head[h]) - want) <= 1      # fixed point vs float may move one row's k by one
        for u in range(M_v):
            assert list(np.nonzero(mask[h, u])[0]) == _brute_topk_row(score[h, u], int(k_head[h]))


def test_mass_rule_equals_the_plain_cumulative_definition_exactly():
    """On rows whose scores are multiples of 2^-10 (so that fixed point loses nothing) the keep count is the plain
    definition - the fewest top-ranked blocks whose scores sum to at least mass x the row total - evaluated in
    exact rational arithmetic.  Rows where some prefix sum sits within two fixed-point units of the target are
    left out (none for the dyadic mass, where the target itself is exact)."""
    from fractions import Fraction
    rng = np.random.default_rng(17)
    M_v = 48
    checked = 0
    for trial in range(300):
        ints = rng.choice(1 << 14, size=M_v, replace=False)               # distinct, so the ranking has no ties
        row = (ints.astype(np.float64) / 1024.0).astype(np.float32)       # exact in fp32: 14 significant bits
        exact = sorted((Fraction(int(i), 1024) for i in ints), reverse=True)
        total = sum(exact)
        for mass in (0.75, 0.5, 0.9, 0.33):
            target = Fraction(mass) * total                                # Fraction(float) is exact
            run, k_def, near = Fraction(0), None, False
            for k, x in enumerate(exact, start=1):
                run += x
                near |= abs(run - target) * (1 << 24) < 2
                if k_def is None and run >= target:
                    k_def = k
            if near and mass not in (0.75, 0.5):
                continue
            assert O.mass_keep_count(row, mass) == k_def, (trial, mass)
            checked += 1
    assert checked >= 1150


def test_mass_row_rule():
    M_v = 40
    score = np.zeros((1, M_v, M_v), dtype=np.float32)
    score[0, :, :] = 1e-3
    score[0, 0, 7] = 10.0                                   # one dominant block: k = floor
    score[0, 1, :] = 0.1                                    # uniform: k = ceil(mass * M_v)
    geo = (0.5 ** np.arange(1, M_v + 1)).astype(np.float32)
    score[0, 2, :] = geo[::-1]                              # geometric: k = 4 for mass 0.9
    mask, k_row = O.select_mass_row(score, 0.9, 0.95)
    assert list(k_row[0, :3]) == [2, 36, 4]
    assert list(np.nonzero(mask[0, 0])[0]) == [0, 7]        # the dominant block, then the lowest-index tie
    assert list(np.nonzero(mask[0, 2])[0]) == [36, 37, 38, 39]
    assert np.array_equal(mask[0].sum(axis=1), k_row[0])
    # against the per-head rule: the head count is the rounded-up mean of the per-row counts (floor applied after)
    rng = np.random.default_rng(9)
    sc = (rng.random((2, M_v, M_v)) ** 5).astype(np.float32)
    _, k_row = O.select_mass_row(sc, 0.8, 1.0 - 1.0 / M_v)  # cap so loose that the floor is one block
    _, k_head = O.select_mass_head(sc, 0.8, 1.0 - 1.0 / M_v)
    assert list(k_head) == [math.ceil(k_row[h].sum() / M_v) for h in range(2)]
