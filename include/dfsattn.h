/*
 * dfsattn.h - C ABI of the DFSAttn attention path for AMD MI355X (gfx950).
 *
 * The library runs the sparse 3D self-attention of a video diffusion transformer as the
 * paper's Algorithm 1 states it: a 3D Hilbert-curve token reorder, hierarchical block
 * scoring, top-k / adaptive block-mask selection, block-sparse attention over the
 * reordered sequence, and the inverse reorder.
 *
 * Conventions shared by every entry point
 *   - `g` points to HOST memory.  Every other pointer is DEVICE memory owned by the caller;
 *     the library allocates nothing, frees nothing and keeps no pointer after a call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; no call synchronises or copies to the host.
 *   - Tensors are dense row-major.  Q, K, V, O are [heads, tokens, d]; a batch dimension
 *     folds into `heads`.  Source ("raster") order has N = T*H*W + n_text tokens, video token
 *     n = (t*H + h)*W + w (Sec. 3.1), text tokens after them.  Reordered tensors have
 *     N_pad = M*B rows: the M_v = ceil(T*H*W/B) video blocks in Hilbert order, zero-padded
 *     at the tail of the last one (Sec. 3.2), then the M_x = ceil(n_text/B) text blocks.
 *   - Return value: DFS_OK or a negative dfs_status.  Arguments are checked on the host
 *     before anything is launched; after an error dfs_last_error() describes it.  A scratch
 *     buffer `ws` must hold at least dfs_workspace_bytes() bytes and be 256-byte aligned;
 *     its contents are undefined afterwards.  Q/K/V/O tensors must be 16-byte aligned (rows move
 *     16 bytes at a time), index, count, score and lse arrays 4-byte aligned: DFS_EINVAL otherwise.
 */
#ifndef DFSATTN_H
#define DFSATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DFS_OK = 0,
  DFS_EINVAL = -1,     /* null pointer, bad enum, bad ratio */
  DFS_ESHAPE = -2,     /* geometry outside what the kernels support */
  DFS_EDTYPE = -3,     /* dtype not supported by this entry point */
  DFS_EWORKSPACE = -4, /* ws missing, misaligned or too small */
  DFS_EHIP = -5        /* a HIP call failed; dfs_last_error() holds its message */
} dfs_status;

typedef enum { DFS_F32 = 0, DFS_BF16 = 1 } dfs_dtype;

typedef enum {
  DFS_SELECT_TOPK = 0,     /* Eq. 9: every query block keeps ceil((1-sparsity)*M_v) key blocks */
  DFS_SELECT_MASS_HEAD = 1, /* per-head keep count from the cumulative score mass (see dfs_select_mask) */
  DFS_SELECT_MASS_ROW = 2   /* per-row keep count from the cumulative score mass */
} dfs_select_mode;

/* Problem geometry (Algorithm 1 inputs; Sec. 3.1 for the token layout). */
typedef struct {
  int32_t T, H, W;   /* latent grid: frames, height, width; each in [1, 512] */
  int32_t n_text;    /* appended tokens that always stay dense (Fig. 1), 0 if none */
  int32_t heads;     /* number of (batch x head) slices */
  int32_t d;         /* head dimension: 64 or 128 */
  int32_t B;         /* block size: 64 or 128 (Sec. 6.1 uses 128) */
  int32_t Bs;        /* sub-block size: divides B, B/Bs in {1,2,4,8} (Table 4) */
} dfs_geom;

/* Sizes that follow from a geometry. */
typedef struct {
  int64_t N_v;    /* T*H*W video tokens */
  int64_t N;      /* N_v + n_text */
  int64_t N_pad;  /* M*B rows of every reordered tensor */
  int32_t M_v;    /* video blocks */
  int32_t M_x;    /* text blocks */
  int32_t M;      /* M_v + M_x */
  int32_t r;      /* sub-blocks per block, B/Bs */
  int32_t M_s;    /* video sub-blocks, M_v*r */
  int32_t bits;   /* bits per axis of the enclosing power-of-two cube */
} dfs_sizes;

typedef enum {
  DFS_ORDER_HILBERT3D = 0, /* the method's order: 3D Hilbert curve over (t,h,w) (Sec. 5.1) */
  DFS_ORDER_RASTER = 1,    /* per-frame row-major, the model's own order */
  DFS_ORDER_HILBERT2D = 2, /* Hilbert order inside each frame, frames in sequence (ablation, Sec. 6.3) */
  DFS_ORDER_BLOCK3D = 3    /* 4x4x4 cubes in raster order of the cubes, raster inside a cube (ablation, Sec. 6.3) */
} dfs_order;

typedef enum {
  DFS_WS_HILBERT_PERM = 0,
  DFS_WS_BLOCK_SCORE = 1,
  DFS_WS_SELECT_MASK = 2,
  DFS_WS_FORWARD = 3,      /* dfs_forward on fp32 tensors */
  DFS_WS_FORWARD_BF16 = 4  /* dfs_forward on bf16 tensors */
} dfs_ws_kind;

/* Validates `g` and fills `out`.  Host only. */
int dfs_geom_sizes(const dfs_geom* g, dfs_sizes* out);

/* Bytes of scratch the given entry point needs for `g` (0 if the geometry is invalid). Host only. */
size_t dfs_workspace_bytes(const dfs_geom* g, int kind);

/* Message of the calling thread's most recent failed call; never NULL. */
const char* dfs_last_error(void);

/* Keep count of DFS_SELECT_TOPK: clamp(ceil((1-sparsity)*M_v - 1e-6), 1, M_v) in double (Eq. 9,
 * with the rounding the paper leaves open).  Host only; returns 0 on invalid arguments. */
int32_t dfs_keep_count(double sparsity, int32_t M_v);

/*
 * Token permutation P (Sec. 5.1; Algorithm 1 step 1).  Video tokens are ordered by the 3D
 * Hilbert index of their cell (t,h,w) in the smallest power-of-two cube holding the grid
 * (Butz curve in Skilling's transpose form, t the most significant axis of each octal digit);
 * text tokens keep their order behind the video blocks.
 *   perm_pad  [N_pad] out  source token of each reordered position, -1 on pad positions
 *   inv       [N]     out  reordered position of each source token
 *   blk_valid [M]     out  real tokens per block (pads are always at a block's tail)
 * Computed once per geometry: the map depends on the grid alone (Sec. 6.3).  ws: DFS_WS_HILBERT_PERM.
 */
int dfs_hilbert_perm(const dfs_geom* g, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * Token permutation for any of the traversal orders of the ablation in Sec. 6.3 (Table 3); with
 * DFS_ORDER_HILBERT3D it is dfs_hilbert_perm.  Same outputs, layout and workspace as dfs_hilbert_perm.
 */
int dfs_token_order(const dfs_geom* g, int order, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * X' = P(X) (Algorithm 1 step 1): x_perm[h, p, :] = x[h, perm_pad[p], :], zeros where
 * perm_pad[p] < 0.   x [heads, N, d] in, x_perm [heads, N_pad, d] out, both of `dtype`.
 */
int dfs_permute(const dfs_geom* g, int dtype, const void* x, const int32_t* perm_pad,
                void* x_perm, void* stream);

/*
 * Hierarchical block score (Sec. 5.2; Algorithm 1 step 2; Eq. 2 and Eq. 8).  Q' and K' are
 * average-pooled over sub-blocks of Bs rows (mean over real rows; a sub-block without real
 * rows is empty), A_hat = row-softmax(Q_hat K_hat^T / sqrt(d)) over the non-empty video
 * sub-blocks, and score[h,u,v] = sum of the r x r entries of A_hat in block pair (u,v).
 * Text blocks are not scored.  Means, softmax and sums are fp32; the logits run on the fp16 matrix cores
 * over a two-term split of the fp32 means, scaled by exact powers of two per four sub-blocks (22 bits per
 * operand: as accurate as an fp32 contraction; an element more than 2^14 times smaller than the largest of its
 * four sub-blocks is kept to 2^-36 of that largest one instead).  Non-finite inputs give non-finite or
 * meaningless scores.
 *   q_perm, k_perm [heads, N_pad, d] in (`dtype`);  score [heads, M_v, M_v] out, fp32.
 * ws: DFS_WS_BLOCK_SCORE (the pooled means and an fp32 array of about heads x M_v x M_s partial log-sums,
 * padded to whole tiles: 0.33 GB at 75 600 tokens x 40 heads).
 */
int dfs_block_score(const dfs_geom* g, int dtype, const void* q_perm, const void* k_perm,
                    float* score, void* ws, size_t ws_bytes, void* stream);

/*
 * Block-mask selection (Eq. 9).  Per (head, query block u) the key blocks are ranked by score,
 * higher first, equal scores by lower index, and the first k are kept.
 *   DFS_SELECT_TOPK:      k = dfs_keep_count(sparsity, M_v) for every head.
 *   DFS_SELECT_MASS_HEAD: per row, k_u = the fewest top blocks whose scores hold a fraction
 *     `mass` of the row total, with scores taken to fixed point floor(clamp(s,0,4096)*2^24) so
 *     that the sums are exact, target ceil(mass*total) in double, k_u >= 1; per head
 *     k_h = max(ceil(mean_u k_u), dfs_keep_count(sparsity, M_v)) with `sparsity` the cap; k_h is
 *     clamped to K_max - M_x.  (This rule is the benchmark's adaptive ratio, not the step
 *     schedule of Sec. 5.3, which is a host policy on `sparsity`.)
 *   DFS_SELECT_MASS_ROW:  every row keeps its own max(k_u, dfs_keep_count(sparsity, M_v)) blocks, clamped to
 *     K_max - M_x; k_head is not written.
 * Text: video query blocks also keep all M_x text key blocks; text query blocks keep all M.
 *   score  [heads, M_v, M_v] in
 *   mask   [heads, M, M] out, uint8 0/1, may be NULL
 *   kv_idx [heads, M, K_max] out: kept key blocks of each query block, ascending; entries at or
 *          beyond the count are unspecified; rows that keep all M blocks are not written
 *   kv_cnt [heads, M] out: number of kept key blocks
 *   k_head [heads] out, may be NULL: the k used for each head
 *   K_max >= k + M_x (TOPK), >= dfs_keep_count(cap) + M_x (MASS_HEAD, MASS_ROW)
 * ws: DFS_WS_SELECT_MASK.
 */
int dfs_select_mask(const dfs_geom* g, const float* score, int mode, double sparsity, double mass,
                    uint8_t* mask, int32_t* kv_idx, int32_t* kv_cnt, int32_t K_max, int32_t* k_head,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * dfs_select_mask for callers that can neither allocate nor pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus ws), same results bit for bit.
 * The scratch of the mass modes (the per-row and per-head keep counts, 4 (heads M_v + heads) bytes) lives in a
 * 1 MiB buffer inside the library, one per GPU, held until the process ends; a geometry that needs more
 * (heads x M_v above about 260 000) is refused with DFS_EWORKSPACE before anything is launched.  The call
 * allocates and frees nothing.  The first call on a device looks up the buffer's device address (no
 * allocation; make that call outside a graph capture).  Every call on a GPU uses that GPU's one buffer, which
 * keeps the last call's contents; nothing in it has to start at zero (every word is written before it is
 * read), but two calls that overlap in time on one GPU, e.g. on two streams, race on it.
 */
int dfs_select_mask_static(const dfs_geom* g, const float* score, int mode, double sparsity, double mass,
                           uint8_t* mask, int32_t* kv_idx, int32_t* kv_cnt, int32_t K_max, int32_t* k_head,
                           void* stream);

/*
 * Block-sparse attention forward over the reordered sequence (Algorithm 1 step 3; Eq. 1 on the
 * kept block pairs).  For a real query position p in block u, the keys are the real positions of
 * the blocks kv_idx[h,u,0..kv_cnt[h,u]) and o_perm[h,p,:] = sum_j softmax_j(scale <q_p,k_j>) v_j
 * with the softmax normalised over those keys.  A query block with kv_cnt == M attends to every
 * block and its kv_idx row is not read; with kv_cnt == 0 its output rows are zero.
 * bf16: products on the matrix cores, fp32 accumulation and softmax, output rounded to bf16.
 * f32:  fp32 throughout.
 *   q_perm, k_perm, v_perm [heads, N_pad, d] in;  o_perm [heads, N_pad, d] out (pad rows unspecified).
 *       Pad rows of k_perm may hold anything (their logits are discarded); pad rows of v_perm must be
 *       finite, e.g. the zeros dfs_permute writes: the bf16 kernel multiplies them by a zero weight.
 *   lse [heads, N_pad] out or NULL: natural-log sum of exp(scale*logit) over the kept keys, fp32-accurate.
 *       (O is normalised by the sum of the weights as rounded to bf16, the weights its numerator uses; when
 *       lse is requested the bf16 kernel keeps the unrounded fp32 sum beside it, at a few per cent of its
 *       speed, because ln of the rounded sum would be off by up to bf16's unit roundoff 2^-8.)
 *   scale: softmax scale, 1/sqrt(d) in the paper.
 * Lists that break the format cannot make the kernels read out of bounds: a count below zero keeps nothing, a
 * count above K_max (and below M) is cut to K_max, a block id outside [0, M) is read as block 0.
 */
int dfs_sparse_attn_fwd(const dfs_geom* g, int dtype, const void* q_perm, const void* k_perm,
                        const void* v_perm, const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max,
                        float scale, void* o_perm, float* lse, void* stream);

/*
 * Variants that read Q, and write O, in SOURCE order through the permutation, so that Q' and O' are never
 * materialised (only K and V take a reorder pass): the query rows are gathered where they are consumed and the
 * attention kernel scatters its output rows.  Results are bit-identical to dfs_permute + the plain call
 * (+ dfs_unperm).  bf16 tensors only.
 *   q [heads, N, d] in, source order;  perm_pad [N_pad] from dfs_hilbert_perm;  o [heads, N, d] out, source order
 *   lse [heads, N_pad] out or NULL, indexed by reordered position as in dfs_sparse_attn_fwd.
 */
int dfs_block_score_src(const dfs_geom* g, int dtype, const void* q, const int32_t* perm_pad, const void* k_perm,
                        float* score, void* ws, size_t ws_bytes, void* stream);
/* As dfs_block_score_src, but K comes in source order as well: the pooling kernel gathers its rows through the
 * permutation and writes them out in the reordered layout on the way, so the call also does the work of
 * dfs_permute for K (pads as zeros, text rows included; k_perm [heads, N_pad, d] out, bit-identical to
 * dfs_permute) and a step that refreshes the mask reorders only V in a pass of its own.  k_perm must not alias k. */
int dfs_block_score_fused(const dfs_geom* g, int dtype, const void* q, const void* k, const int32_t* perm_pad,
                          void* k_perm, float* score, void* ws, size_t ws_bytes, void* stream);
int dfs_sparse_attn_fwd_src(const dfs_geom* g, int dtype, const void* q, const int32_t* perm_pad, const void* k_perm,
                            const void* v_perm, const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale,
                            void* o, float* lse, void* stream);

/*
 * O = P^{-1}(O') (Algorithm 1 step 3, last line): o[h, n, :] = o_perm[h, inv[n], :].
 *   o_perm [heads, N_pad, d] in, o [heads, N, d] out.
 */
int dfs_unperm(const dfs_geom* g, int dtype, const void* o_perm, const int32_t* inv, void* o, void* stream);

/*
 * Mask state of one attention layer that survives across diffusion steps (Sec. 5.3): the caller
 * owns the buffers and passes them to every step.
 */
typedef struct {
  int32_t* kv_idx;   /* [heads, M, K_max] */
  int32_t* kv_cnt;   /* [heads, M] */
  uint8_t* mask;     /* [heads, M, M] or NULL */
  int32_t* k_head;   /* [heads] or NULL */
  int32_t K_max;
} dfs_mask_state;

/*
 * One call of Algorithm 1 for one layer: reorder Q, K, V; if `refresh` is non-zero recompute the
 * block mask into `st` (scoring + selection as above), otherwise reuse it (Sec. 5.3: masks are
 * refreshed every Delta steps, outputs are recomputed every step); block-sparse attention; inverse
 * reorder.  perm_pad / inv come from dfs_hilbert_perm.
 *   q, k, v [heads, N, d] in;  o [heads, N, d] out.   ws: DFS_WS_FORWARD (f32) or DFS_WS_FORWARD_BF16.
 */
int dfs_forward(const dfs_geom* g, int dtype, const void* q, const void* k, const void* v,
                const int32_t* perm_pad, const int32_t* inv, int refresh, int mode, double sparsity,
                double mass, dfs_mask_state* st, float scale, void* o, void* ws, size_t ws_bytes,
                void* stream);

/*
 * Attention recall (Eq. 3): recall[h] = ||A * M||_1 / ||A||_1, the mean over the real query rows of the
 * attention mass that falls on kept keys, from the log-sum-exp of a run under the mask and of a run with
 * all blocks kept: per row exp(lse_sparse - lse_dense).  The quality proxy of Sec. 3.2 / Fig. 3.
 *   lse_sparse, lse_dense [heads, N_pad] in (from dfs_sparse_attn_fwd);  recall [heads] out, fp32.
 */
int dfs_recall(const dfs_geom* g, const float* lse_sparse, const float* lse_dense, float* recall, void* stream);

/*
 * The paper's step schedule (Sec. 6.1 "Implementation details", App. B; Algorithm 1 for the refresh).  Host only.
 * Steps of the first quarter (t < total_steps/4) run dense attention (*dense = 1).  After that the keep ratio
 * starts at 0.3 and drops by 0.1 every further quarter (*sparsity = 0.7, 0.8, 0.9: about 80 % on average).
 * *refresh = 1 when t is a multiple of delta (12 in the paper for 50 steps), when no mask exists yet
 * (cached_keep < 0) or when the cached mask was built for another keep ratio (cached_keep != 1 - *sparsity);
 * the last two conditions are readings the paper leaves open.
 */
int dfs_schedule(int32_t total_steps, int32_t t, int32_t delta, double cached_keep, int32_t* dense, int32_t* refresh,
                 double* sparsity);

/*
 * Diagnostic for measurements, not part of the method: while `counters` (device memory, 3 x uint64, zeroed by
 * the caller) is set, every work-group of the bf16 attention kernel adds to counters[0] the shader-clock
 * cycles and to counters[1] the constant-rate timer ticks (100 MHz) between its start and its end, and 1 to
 * counters[2].  counters[0] / counters[1] x 100 MHz is the shader clock the kernel ran at, which on this chip
 * sits well below the nominal 2.4 GHz under matrix load.  NULL switches it off (the default).  This is
 * process-wide state that EVERY later launch of the bf16 attention kernel reads, from any thread and on any
 * stream: not thread-safe; the buffer (8-byte aligned) must stay valid until it is switched off again.
 */
int dfs_attn_clock_probe(uint64_t* counters);

/*
 * Measurement probes, not part of the method: what the chip sustains, to set beside the nominal peaks.
 * dfs_probe_mfma launches `work_groups` x 4 waves that run `iters` x 4 independent v_mfma_f32_32x32x16_bf16
 * (32768 flop each per wave) and nothing else; sink [work_groups * 256] fp32 out (device);
 * counters (device, 2 x uint64, zeroed by the caller, or NULL) receives work-group 0's shader-clock cycles and
 * 100 MHz ticks.  dfs_probe_copy copies `bytes` (a multiple of 16, 16-byte aligned device pointers) with
 * 16 bytes per lane.  dfs_probe_read launches `work_groups` x 256 threads that each read `pieces_per_wg`
 * 64 KB pieces of the region src[0, bytes) (a multiple of 64 KB, 16-byte aligned) at seeded pseudo-random piece
 * indices and nothing else: read-only traffic of the shape of the attention kernel's tile loads; sink (device,
 * one uint32) is written only for one particular checksum.  Time them with events on `stream`.
 */
int dfs_probe_mfma(int32_t work_groups, int32_t iters, float* sink, uint64_t* counters, void* stream);
int dfs_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
int dfs_probe_read(const void* src, size_t bytes, int32_t work_groups, int32_t pieces_per_wg, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DFSATTN_H */
