"""CPU oracle for the DFSAttn attention path.  TEST INFRASTRUCTURE ONLY.

A plain, slow numpy/fp64 statement of what each step of the paper's Algorithm 1
computes.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does, and this file imports nothing of the HIP
path.  Every function names the passage it follows.  All floating point is fp64
on exactly up-converted inputs; all index work is exact integer arithmetic.

Readings taken where the paper is silent (each also listed in the design notes):
  * which 3D Hilbert curve, and non-cubic grids      -> hilbert_key / hilbert_perm
  * padding inside the pooled sub-blocks              -> pool
  * rounding of gamma*M, ties, text tokens            -> select_topk
  * the cumulative-mass adaptive ratio (not the paper's schedule) -> select_mass_head
  * masked softmax renormalised over the kept set     -> sparse_attn

Pinned by tests/test_oracle_*.py (run without a GPU).  Nothing here is "parity
unpinned".
"""
from __future__ import annotations

import math

import numpy as np

# ----------------------------------------------------------------------------------------
# Step 1 - 3D Hilbert curve token order (Sec. 5.1; Algorithm 1 step 1)
# ----------------------------------------------------------------------------------------


def cube_bits(T: int, H: int, W: int) -> int:
    """Bits per axis of the smallest power-of-two cube that holds the T x H x W grid."""
    return max(1, int(max(T, H, W) - 1).bit_length())


def hilbert_key_nd(coords, b: int):
    """Hilbert index of cells in the cube [0,2^b)^n, n = len(coords) (Sec. 5.1 for n = 3).

    The paper asks for a 3D Hilbert curve without fixing which of them.  The reading:
    Skilling's transpose form of the Butz curve with the first coordinate the most significant.
    Working from the coarsest bit downward the coordinates are un-rotated (A), then Gray-decoded
    (B), and the n b-bit words are read as b digits of n bits with x0 the high bit of each (C).
    """
    n = len(coords)
    x = [np.array(c, dtype=np.int64).copy() for c in coords]
    # (A) undo the sub-cube rotations, coarsest level first
    Q = 1 << (b - 1)
    while Q > 1:
        P = Q - 1
        for i in range(n):
            hi = (x[i] & Q) != 0
            # bit set: reflect the low bits of x0; clear: exchange low bits of x0 and xi
            s = np.where(hi, 0, (x[0] ^ x[i]) & P)
            x[0] = np.where(hi, x[0] ^ P, x[0] ^ s)
            x[i] = x[i] ^ s
        Q >>= 1
    # (B) Gray decode across the axes
    for i in range(1, n):
        x[i] = x[i] ^ x[i - 1]
    s = np.zeros_like(x[0])
    Q = 1 << (b - 1)
    while Q > 1:
        s = np.where((x[n - 1] & Q) != 0, s ^ (Q - 1), s)
        Q >>= 1
    x = [xi ^ s for xi in x]
    # (C) interleave: digit j = sum_i bit_j(x_i) << (n-1-i)
    key = np.zeros_like(x[0])
    for j in range(b - 1, -1, -1):
        digit = np.zeros_like(x[0])
        for i in range(n):
            digit = (digit << 1) | ((x[i] >> j) & 1)
        key = (key << n) | digit
    return key


def hilbert_key(t, h, w, b: int):
    """3D Hilbert index of the cells (t,h,w) in the cube [0,2^b)^3, axes (x0,x1,x2) = (t,h,w)."""
    return hilbert_key_nd([t, h, w], b)


ORDERS = ("hilbert3d", "raster", "hilbert2d", "block3d")


def order_keys(kind: str, T: int, H: int, W: int):
    """Sort key of every video token (raster index n) under a traversal order.

    hilbert3d: the method's order (Sec. 5.1).  The others are the orderings of the ablation
    (Sec. 6.3, Table 3): raster = per-frame row-major (the model's own order); hilbert2d = Hilbert
    order inside each frame, frames in sequence; block3d = 4x4x4 cubes in raster order of the
    cubes, raster traversal inside a cube.  Keys are distinct within a kind.
    """
    n = np.arange(T * H * W, dtype=np.int64)
    t, h, w = n // (H * W), (n // W) % H, n % W
    if kind == "hilbert3d":
        return hilbert_key(t, h, w, cube_bits(T, H, W))
    if kind == "raster":
        return n
    if kind == "hilbert2d":
        b2 = cube_bits(1, H, W)
        return (t << (2 * b2)) | hilbert_key_nd([h, w], b2)
    if kind == "block3d":
        ch, cw = -(-H // 4), -(-W // 4)
        cube = ((t // 4) * ch + h // 4) * cw + w // 4
        return cube * 64 + ((t % 4) * 4 + h % 4) * 4 + w % 4
    raise ValueError(kind)


def token_order(kind: str, T: int, H: int, W: int, n_text: int, B: int):
    """Permutation and padded block layout for a traversal order (see hilbert_perm for the layout)."""
    N_v = T * H * W
    order = np.argsort(order_keys(kind, T, H, W), kind="stable")
    M_v = -(-N_v // B)
    M_x = -(-n_text // B)
    M = M_v + M_x
    perm_pad = np.full(M * B, -1, dtype=np.int32)
    perm_pad[:N_v] = order
    perm_pad[M_v * B: M_v * B + n_text] = N_v + np.arange(n_text)
    inv = np.empty(N_v + n_text, dtype=np.int32)
    pos = np.nonzero(perm_pad >= 0)[0]
    inv[perm_pad[pos]] = pos
    blk_valid = (perm_pad.reshape(M, B) >= 0).sum(axis=1).astype(np.int32)
    return perm_pad, inv, blk_valid


def hilbert_perm(T: int, H: int, W: int, n_text: int, B: int):
    """Token permutation P of Algorithm 1 step 1 and the padded block layout (Sec. 3.2).

    Video token n = (t*H + h)*W + w (per-frame row-major, Sec. 3.1).  Video tokens are
    ordered by ascending Hilbert key of their cell; the sequence is padded to a multiple
    of B (Sec. 3.2); text tokens keep their order in blocks of their own after the video
    blocks.  Returns
      perm_pad[N_pad]  source token of each position, -1 on pad positions
      inv[N]           position of each source token
      blk_valid[M]     number of real tokens in each block (pads sit at a block's tail)
    """
    N_v = T * H * W
    b = cube_bits(T, H, W)
    n = np.arange(N_v, dtype=np.int64)
    keys = hilbert_key(n // (H * W), (n // W) % H, n % W, b)
    order = np.argsort(keys, kind="stable")            # keys are distinct
    M_v = -(-N_v // B)
    M_x = -(-n_text // B)
    M = M_v + M_x
    perm_pad = np.full(M * B, -1, dtype=np.int32)
    perm_pad[:N_v] = order
    perm_pad[M_v * B: M_v * B + n_text] = N_v + np.arange(n_text)
    inv = np.empty(N_v + n_text, dtype=np.int32)
    pos = np.nonzero(perm_pad >= 0)[0]
    inv[perm_pad[pos]] = pos
    blk_valid = (perm_pad.reshape(M, B) >= 0).sum(axis=1).astype(np.int32)
    return perm_pad, inv, blk_valid


def permute(x: np.ndarray, perm_pad: np.ndarray) -> np.ndarray:
    """X' = P(X) (Algorithm 1 step 1): row gather, zero rows on pad positions.  x: [heads,N,d]."""
    out = np.zeros((x.shape[0], perm_pad.shape[0], x.shape[2]), dtype=x.dtype)
    real = perm_pad >= 0
    out[:, real, :] = x[:, perm_pad[real], :]
    return out


def unpermute(o_perm: np.ndarray, inv: np.ndarray) -> np.ndarray:
    """O = P^{-1}(O') (Algorithm 1 step 3): source token n reads position inv[n]."""
    return o_perm[:, inv, :]


# ----------------------------------------------------------------------------------------
# Step 2 - hierarchical block scoring (Sec. 5.2; Algorithm 1 step 2; Eq. 8)
# ----------------------------------------------------------------------------------------


def pool(x_perm: np.ndarray, N_v: int, Bs: int, M_s: int):
    """AvgPool(X', B_s) over the video segment (Algorithm 1 step 2).

    x_perm: [heads, N_pad, d] fp64.  Sub-block s covers positions [s*Bs, (s+1)*Bs); only
    positions < N_v are real.  The mean is over real positions (reading: the paper does not
    say how padding enters the pool); a sub-block with no real position is empty.
    Returns (centroids [heads, M_s, d], count [M_s]).
    """
    heads, _, d = x_perm.shape
    cen = np.zeros((heads, M_s, d), dtype=np.float64)
    cnt = np.zeros(M_s, dtype=np.int64)
    for s in range(M_s):
        lo, hi = s * Bs, min((s + 1) * Bs, N_v)
        if hi > lo:
            cnt[s] = hi - lo
            cen[:, s, :] = x_perm[:, lo:hi, :].sum(axis=1) / float(hi - lo)
    return cen, cnt


def subblock_softmax(q_hat: np.ndarray, k_hat: np.ndarray, cnt: np.ndarray, d: int) -> np.ndarray:
    """A_hat = softmax(Q_hat K_hat^T / sqrt(d)) (Eq. 2; Algorithm 1 step 2), one head.

    Rows and columns are sub-blocks; empty sub-blocks get probability 0 as columns and an
    all-zero row as queries.
    """
    logits = (q_hat @ k_hat.T) / math.sqrt(d)
    live = cnt > 0
    logits[:, ~live] = -np.inf
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    a = e / e.sum(axis=1, keepdims=True)
    a[~live, :] = 0.0
    return a


def aggregate(a_hat: np.ndarray, r: int) -> np.ndarray:
    """S_hat[u,v] = sum of the r x r sub-block scores of block pair (u,v) (Eq. 8)."""
    M_s = a_hat.shape[0]
    M_v = M_s // r
    return a_hat.reshape(M_v, r, M_v, r).sum(axis=(1, 3))


def block_score(q_perm: np.ndarray, k_perm: np.ndarray, N_v: int, B: int, Bs: int) -> np.ndarray:
    """Hierarchical block score S_hat [heads, M_v, M_v] (Sec. 5.2), fp64."""
    heads, _, d = q_perm.shape
    r = B // Bs
    M_v = -(-N_v // B)
    M_s = M_v * r
    q_hat, cnt = pool(q_perm, N_v, Bs, M_s)
    k_hat, _ = pool(k_perm, N_v, Bs, M_s)
    out = np.empty((heads, M_v, M_v), dtype=np.float64)
    for h in range(heads):
        out[h] = aggregate(subblock_softmax(q_hat[h], k_hat[h], cnt, d), r)
    return out


# ----------------------------------------------------------------------------------------
# Step 2 (cont.) - block selection (Eq. 9) and the adaptive ratio
# ----------------------------------------------------------------------------------------


def keep_count(sparsity: float, M_v: int) -> int:
    """Number of key blocks kept per query block: ceil(gamma*M_v), gamma = 1 - sparsity (Eq. 9).

    Reading: the paper writes "gamma M" without a rounding rule; rounding up never drops
    more than asked, the 1e-6 guards an exact product against representation error, and at
    least one block is always kept.
    """
    gamma = 1.0 - float(sparsity)
    return int(min(max(math.ceil(gamma * M_v - 1e-6), 1), M_v))


def _rank_order(row: np.ndarray) -> np.ndarray:
    """Columns of a score row from best to worst: higher score first, ties by lower index."""
    return np.lexsort((np.arange(row.shape[0]), -row))


def build_mask(keep_cols, M_v: int, M_x: int) -> np.ndarray:
    """Block mask [M, M] of one head from the kept video columns of each video query block.

    Text blocks (Fig. 1: text stays dense): every video query block also keeps all text
    key blocks; text query blocks keep every key block.
    """
    M = M_v + M_x
    mask = np.zeros((M, M), dtype=np.uint8)
    for u in range(M_v):
        mask[u, keep_cols[u]] = 1
    mask[:M_v, M_v:] = 1
    mask[M_v:, :] = 1
    return mask


def select_topk(score: np.ndarray, sparsity: float, M_x: int = 0):
    """Top-(gamma M) key blocks per query block (Eq. 9).  score: [heads, M_v, M_v].

    Returns (mask [heads, M, M] uint8, k).  Scores are compared as given (the caller passes
    fp32 scores when the decision is to be taken in fp32).
    """
    heads, M_v, _ = score.shape
    k = keep_count(sparsity, M_v)
    mask = np.empty((heads, M_v + M_x, M_v + M_x), dtype=np.uint8)
    for h in range(heads):
        mask[h] = build_mask([_rank_order(score[h, u])[:k] for u in range(M_v)], M_v, M_x)
    return mask, k


MASS_FRAC_BITS = 24


def mass_keep_count(row: np.ndarray, mass: float) -> int:
    """Smallest k whose top-k scores hold at least `mass` of the row's total score.

    Reading of "keep cumulative block-score mass >= mass": scores are taken to fixed point,
    q = floor(s * 2^24) for s clamped to [0, 4096], so that the sums are exact integers and
    do not depend on summation order; the target is ceil(mass * total) evaluated in fp64
    (total < 2^53 is exact); k is at least 1.
    """
    s = np.clip(row.astype(np.float64), 0.0, 4096.0)
    q = np.floor(s * float(1 << MASS_FRAC_BITS)).astype(np.int64)
    total = int(q.sum())
    target = int(math.ceil(float(mass) * float(total)))
    if target <= 0:
        return 1
    run = 0
    for k, j in enumerate(_rank_order(row), start=1):
        run += int(q[j])
        if run >= target:
            return k
    return row.shape[0]


def select_mass_head(score: np.ndarray, mass: float, cap_sparsity: float, M_x: int = 0):
    """Adaptive per-head ratio: each head keeps k_h blocks per query block, where k_h is the
    rounded-up mean over its query blocks of mass_keep_count, never below the keep count at
    the sparsity cap.  (This adaptive rule is the benchmark configuration's, not the paper's
    step schedule of Sec. 5.3.)  Returns (mask, k_head [heads]).
    """
    heads, M_v, _ = score.shape
    k_floor = keep_count(cap_sparsity, M_v)
    mask = np.empty((heads, M_v + M_x, M_v + M_x), dtype=np.uint8)
    k_head = np.empty(heads, dtype=np.int32)
    for h in range(heads):
        ksum = sum(mass_keep_count(score[h, u], mass) for u in range(M_v))
        k_h = max(-(-ksum // M_v), k_floor)
        k_head[h] = k_h
        mask[h] = build_mask([_rank_order(score[h, u])[:k_h] for u in range(M_v)], M_v, M_x)
    return mask, k_head


def select_mass_row(score: np.ndarray, mass: float, cap_sparsity: float, M_x: int = 0):
    """Adaptive per-row ratio: every query block keeps its own mass_keep_count blocks, never fewer than the
    keep count at the sparsity cap.  (The per-row form of select_mass_head.)  Returns (mask, k_row [heads, M_v])."""
    heads, M_v, _ = score.shape
    k_floor = keep_count(cap_sparsity, M_v)
    mask = np.empty((heads, M_v + M_x, M_v + M_x), dtype=np.uint8)
    k_row = np.empty((heads, M_v), dtype=np.int32)
    for h in range(heads):
        cols = []
        for u in range(M_v):
            k_row[h, u] = max(mass_keep_count(score[h, u], mass), k_floor)
            cols.append(_rank_order(score[h, u])[:k_row[h, u]])
        mask[h] = build_mask(cols, M_v, M_x)
    return mask, k_row


def mask_to_lists(mask: np.ndarray, K_max: int):
    """kv_idx [heads, M, K_max] (ascending kept columns, -1 beyond the count) and kv_cnt.
    K_max must hold the longest row."""
    heads, M, _ = mask.shape
    kv_idx = np.full((heads, M, K_max), -1, dtype=np.int32)
    kv_cnt = np.zeros((heads, M), dtype=np.int32)
    for h in range(heads):
        for u in range(M):
            cols = np.nonzero(mask[h, u])[0]
            kv_cnt[h, u] = cols.shape[0]
            kv_idx[h, u, :cols.shape[0]] = cols
    return kv_idx, kv_cnt


# ----------------------------------------------------------------------------------------
# Step 3 - attention (Eq. 1; block-sparse form of Sec. 3.2 as executed in Sec. 5.2)
# ----------------------------------------------------------------------------------------


def dense_attn(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """O = softmax(Q K^T / sqrt(d)) V (Eq. 1), one head, fp64."""
    d = q.shape[1]
    s = (q @ k.T) / math.sqrt(d)
    s -= s.max(axis=1, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=1, keepdims=True)) @ v


def sparse_attn_block(q_perm, k_perm, v_perm, cols, blk_valid, B: int, u: int, scale: float):
    """Output rows and log-sum-exp of query block u of one head, given its kept key blocks.

    A query attends to the real tokens of the kept key blocks only, and the softmax is
    normalised over that set: the method runs a FlashAttention kernel on the kept block
    pairs (Sec. 5.2, last paragraph), which renormalises.  Returns (o [B, d], lse [B]);
    pad query rows are computed like any other and are ignored by callers.
    """
    keys = np.concatenate([np.arange(c * B, c * B + blk_valid[c]) for c in cols]) \
        if len(cols) else np.zeros(0, dtype=np.int64)
    qb = q_perm[u * B:(u + 1) * B]
    if keys.size == 0:
        return np.zeros_like(qb), np.full(B, -np.inf)
    s = (qb @ k_perm[keys].T) * scale
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    z = p.sum(axis=1, keepdims=True)
    return (p / z) @ v_perm[keys], (m + np.log(z))[:, 0]


def sparse_attn(q_perm, k_perm, v_perm, mask, blk_valid, B: int, scale=None, q_blocks=None):
    """Block-sparse attention over the reordered sequence (Algorithm 1 step 3).

    q_perm, k_perm, v_perm: [heads, N_pad, d] fp64; mask: [heads, M, M].  Returns
    (o_perm [heads, N_pad, d], lse [heads, N_pad]); only the query blocks in `q_blocks`
    (default: all) are filled, the others are NaN.
    """
    heads, N_pad, d = q_perm.shape
    M = N_pad // B
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    o = np.full((heads, N_pad, d), np.nan)
    lse = np.full((heads, N_pad), np.nan)
    for h in range(heads):
        for u in (range(M) if q_blocks is None else q_blocks):
            cols = np.nonzero(mask[h, u])[0]
            o[h, u * B:(u + 1) * B], lse[h, u * B:(u + 1) * B] = sparse_attn_block(
                q_perm[h], k_perm[h], v_perm[h], cols, blk_valid, B, u, scale)
    return o, lse


# ----------------------------------------------------------------------------------------
# Algorithm 1 end to end, with the cached mask (Sec. 5.3)
# ----------------------------------------------------------------------------------------


class DFSAttnOracle:
    """Algorithm 1 for one attention layer: the permutation is fixed per geometry, the block
    mask is recomputed when t is a multiple of delta and reused otherwise, and the outputs
    are recomputed at every step (Sec. 5.3)."""

    def __init__(self, T, H, W, n_text, B, Bs, delta=1, score_dtype=np.float64):
        self.T, self.H, self.W, self.n_text, self.B, self.Bs = T, H, W, n_text, B, Bs
        self.N_v = T * H * W
        self.M_x = -(-n_text // B)
        self.delta = delta
        self.score_dtype = score_dtype
        self.perm_pad, self.inv, self.blk_valid = hilbert_perm(T, H, W, n_text, B)
        self.mask = None

    def step(self, q, k, v, t, sparsity=None, mass=None, cap=0.95):
        """q, k, v: [heads, N, d] fp64 in raster order.  Returns O [heads, N, d]."""
        qp, kp, vp = (permute(x, self.perm_pad) for x in (q, k, v))
        if self.mask is None or t % self.delta == 0:
            score = block_score(qp, kp, self.N_v, self.B, self.Bs).astype(self.score_dtype)
            if mass is not None:
                self.mask, _ = select_mass_head(score, mass, cap, self.M_x)
            else:
                self.mask, _ = select_topk(score, sparsity, self.M_x)
        o_perm, _ = sparse_attn(qp, kp, vp, self.mask, self.blk_valid, self.B)
        return unpermute(o_perm, self.inv)


# ----------------------------------------------------------------------------------------
# Attention recall (Eq. 3) and the paper's step schedule (Sec. 5.3, Sec. 6.1, App. B)
# ----------------------------------------------------------------------------------------


def attention_recall(q_perm, k_perm, mask, blk_valid, B: int):
    """R = ||A * M||_1 / ||A||_1 (Eq. 3) per head, with M the token-level form of the block mask and
    A the full attention matrix of Eq. 1 over the real tokens: the mean over real query rows of the
    attention mass that falls on kept key blocks.  q_perm, k_perm: [heads, N_pad, d] fp64."""
    heads, N_pad, d = q_perm.shape
    M = N_pad // B
    real = np.concatenate([np.arange(u * B, u * B + blk_valid[u]) for u in range(M)])
    blk_of = real // B
    out = np.empty(heads)
    for h in range(heads):
        s = (q_perm[h][real] @ k_perm[h][real].T) / math.sqrt(d)
        a = np.exp(s - s.max(axis=1, keepdims=True))
        a /= a.sum(axis=1, keepdims=True)
        keep = mask[h][blk_of][:, blk_of].astype(bool)     # token-level mask
        out[h] = (a * keep).sum() / a.sum()
    return out


def paper_schedule(total_steps: int, t: int, delta: int = 12, dense_frac: float = 0.25, keep0: float = 0.3,
                   keep_step: float = 0.1, cached_keep=None):
    """What step t of a sampling run does (Sec. 6.1 "Implementation details", App. B; Alg. 1 for the refresh).

    Steps in the first quarter run dense attention.  After that the keep ratio starts at keep0 and drops by
    keep_step every further quarter (0.3 -> 0.2 -> 0.1, about 80 % mean sparsity).  The mask is recomputed
    when t is a multiple of delta (Alg. 1) and, readings the paper leaves open, when no mask exists yet
    (first sparse step) or when the cached mask was built for another keep ratio (`cached_keep`).
    Returns (dense, refresh, sparsity).
    """
    quarter = min(int(math.floor(t / (dense_frac * total_steps) + 1e-9)), int(round(1 / dense_frac)) - 1)
    if quarter == 0:
        return True, False, 0.0
    keep = keep0 - keep_step * (quarter - 1)
    refresh = (t % delta == 0) or cached_keep is None or abs(cached_keep - keep) > 1e-12
    return False, refresh, 1.0 - keep
