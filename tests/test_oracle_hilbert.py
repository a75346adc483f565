"""Pins for the oracle's Hilbert order and padded layout (paper Sec. 5.1, Sec. 3.2).

The curve is pinned by what the mathematics fixes: it visits every cell of a power-of-two
cube once, consecutive cells are unit steps apart, it starts at the origin and ends at the
far corner of the first axis, level 1 is the reflected Gray code, the top digit of a level-b
key is the level-1 key of the cell's octant, plus hand-worked values (tests/golden).
"""
import os

import numpy as np
import pytest

from oracle import dfs_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hilbert_pins.txt")


def _cube(b):
    n = 1 << b
    t, h, w = np.meshgrid(np.arange(n), np.arange(n), np.arange(n), indexing="ij")
    return t.ravel(), h.ravel(), w.ravel()


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5])
def test_bijection_and_unit_steps(b):
    t, h, w = _cube(b)
    key = O.hilbert_key(t, h, w, b)
    assert np.array_equal(np.sort(key), np.arange(8 ** b))
    order = np.argsort(key)
    cells = np.stack([t[order], h[order], w[order]], axis=1)
    step = np.abs(np.diff(cells, axis=0)).sum(axis=1)
    assert np.all(step == 1)
    assert tuple(cells[0]) == (0, 0, 0)
    assert tuple(cells[-1]) == ((1 << b) - 1, 0, 0)


def test_level_one_is_gray_code():
    t, h, w = _cube(1)
    order = np.argsort(O.hilbert_key(t, h, w, 1))
    got = [(int(t[i]), int(h[i]), int(w[i])) for i in order]
    assert got == [(0, 0, 0), (0, 0, 1), (0, 1, 1), (0, 1, 0), (1, 1, 0), (1, 1, 1), (1, 0, 1), (1, 0, 0)]


@pytest.mark.parametrize("b", [2, 3, 4])
def test_octants_are_visited_in_level_one_order(b):
    t, h, w = _cube(b)
    key = O.hilbert_key(t, h, w, b)
    top = O.hilbert_key(t >> (b - 1), h >> (b - 1), w >> (b - 1), 1)
    assert np.array_equal(key >> (3 * (b - 1)), top)


def _gold():
    keys, cells, perms = [], None, []
    for line in open(GOLD):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "key":
            keys.append(tuple(int(x) for x in f[1:]))
        elif f[0] == "cells":
            cells = np.array([int(x) for x in f[1:]]).reshape(8, 3)
        elif f[0] == "perm":
            perms.append((tuple(int(x) for x in f[1:4]), [int(x) for x in f[4:12]], int(f[12]), f[13]))
    return keys, cells, perms


def test_hand_worked_keys():
    keys, cells, _ = _gold()
    for t, h, w, b, val in keys:
        assert int(O.hilbert_key(t, h, w, b)) == val
    t, h, w = _cube(2)
    order = np.argsort(O.hilbert_key(t, h, w, 2))[:8]
    assert np.array_equal(np.stack([t[order], h[order], w[order]], axis=1), cells)


def _fnv1a64(data: bytes) -> str:
    h = 0xCBF29CE484222325
    for byte in data:
        h = ((h ^ byte) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return "%016x" % h


def test_config_grids_match_recorded_digests():
    _, _, perms = _gold()
    for (T, H, W), first, last, digest in perms:
        perm_pad, _, _ = O.hilbert_perm(T, H, W, 0, 128)
        pv = perm_pad[:T * H * W]
        assert list(pv[:8]) == first
        assert int(pv[-1]) == last
        assert _fnv1a64(pv.astype("<i4").tobytes()) == digest


@pytest.mark.parametrize("T,H,W,n_text,B", [(4, 8, 8, 0, 64), (3, 5, 7, 0, 16), (5, 6, 9, 10, 32), (2, 2, 2, 33, 16)])
def test_padded_layout(T, H, W, n_text, B):
    perm_pad, inv, blk_valid = O.hilbert_perm(T, H, W, n_text, B)
    N_v, N = T * H * W, T * H * W + n_text
    M_v, M_x = -(-N_v // B), -(-n_text // B)
    assert perm_pad.shape == ((M_v + M_x) * B,) and inv.shape == (N,) and blk_valid.shape == (M_v + M_x,)
    # every source token appears exactly once; pads are -1
    real = perm_pad[perm_pad >= 0]
    assert np.array_equal(np.sort(real), np.arange(N))
    assert np.array_equal(perm_pad[inv], np.arange(N))
    # video tokens fill [0, N_v), text tokens start at the first text block, in order
    assert np.all(perm_pad[:N_v] < N_v) and np.all(perm_pad[:N_v] >= 0)
    assert np.all(perm_pad[N_v:M_v * B] == -1)
    assert np.array_equal(perm_pad[M_v * B:M_v * B + n_text], N_v + np.arange(n_text))
    assert np.all(perm_pad[M_v * B + n_text:] == -1)
    # pads only at block tails, counts add up
    for blk in range(M_v + M_x):
        row = perm_pad[blk * B:(blk + 1) * B]
        assert np.all(row[:blk_valid[blk]] >= 0) and np.all(row[blk_valid[blk]:] == -1)
    assert blk_valid.sum() == N
    # the video order is ascending in Hilbert key of the enclosing cube
    b = O.cube_bits(T, H, W)
    n = perm_pad[:N_v].astype(np.int64)
    key = O.hilbert_key(n // (H * W), (n // W) % H, n % W, b)
    assert np.all(np.diff(key) > 0)


def test_locality_of_config_grid():
    # On the 4x8x8 slab every step of the order is a unit step (the slab is two 4x4x4... cubes
    # traversed contiguously); on a non-power-of-two grid most steps still are.
    perm_pad, _, _ = O.hilbert_perm(4, 8, 8, 0, 64)
    n = perm_pad.astype(np.int64)
    cells = np.stack([n // 64, (n // 8) % 8, n % 8], axis=1)
    assert np.all(np.abs(np.diff(cells, axis=0)).sum(axis=1) == 1)
    perm_pad, _, _ = O.hilbert_perm(13, 30, 45, 0, 128)
    n = perm_pad[:13 * 30 * 45].astype(np.int64)
    cells = np.stack([n // 1350, (n // 45) % 30, n % 45], axis=1)
    unit = (np.abs(np.diff(cells, axis=0)).sum(axis=1) == 1).mean()
    assert unit > 0.97


def test_permute_roundtrip():
    rng = np.random.default_rng(0)
    perm_pad, inv, _ = O.hilbert_perm(3, 5, 7, 6, 16)
    x = rng.standard_normal((2, 3 * 5 * 7 + 6, 4))
    xp = O.permute(x, perm_pad)
    assert np.all(xp[:, perm_pad < 0, :] == 0)
    assert np.array_equal(O.unpermute(xp, inv), x)
