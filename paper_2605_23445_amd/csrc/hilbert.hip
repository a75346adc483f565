// Token permutation by 3D Hilbert index (paper Sec. 5.1; Algorithm 1 step 1) and by the other
// traversal orders of the ablation in Sec. 6.3.
//
// Keys are ranked without a sort: every token sets the bit of its key in a bitmap over the key
// space (for the Hilbert order: the cells of the enclosing 2^b cube), a prefix sum over the bitmap
// words turns a key into its rank among the keys in use, and every token then writes itself at its
// rank.  Integer work only; run once per geometry.
#include "common.h"

namespace dfs {

// Hilbert index of a cell in [0,2^b)^N: Butz curve in Skilling's transpose form.  Level by level from
// the coarsest bit, a set bit of an axis reflects the lower bits of x0 and a clear bit exchanges the
// lower bits of x0 with that axis; a Gray decode across the axes follows; the N words are then read as
// b digits of N bits with x0 the high bit.
template <int N>
__device__ __forceinline__ uint32_t hilbert_index(uint32_t (&x)[N], int b) {
  for (uint32_t q = 1u << (b - 1); q > 1; q >>= 1) {
    const uint32_t low = q - 1;
#pragma unroll
    for (int a = 0; a < N; ++a) {
      if (x[a] & q) {
        x[0] ^= low;
      } else {
        const uint32_t swap = (x[0] ^ x[a]) & low;
        x[0] ^= swap;
        x[a] ^= swap;
      }
    }
  }
#pragma unroll
  for (int a = 1; a < N; ++a) x[a] ^= x[a - 1];
  uint32_t fix = 0;
  for (uint32_t q = 1u << (b - 1); q > 1; q >>= 1)
    if (x[N - 1] & q) fix ^= q - 1;
#pragma unroll
  for (int a = 0; a < N; ++a) x[a] ^= fix;
  uint32_t key = 0;
  for (int j = b - 1; j >= 0; --j) {
    uint32_t digit = 0;
#pragma unroll
    for (int a = 0; a < N; ++a) digit = (digit << 1) | ((x[a] >> j) & 1u);
    key = (key << N) | digit;
  }
  return key;
}

// Sort key of video token n under a traversal order (distinct keys within an order):
//   hilbert3d  3D Hilbert index of (t,h,w) in the enclosing cube (Sec. 5.1)
//   raster     n itself (per-frame row-major, the model's own order)
//   hilbert2d  frame index, then the 2D Hilbert index of (h,w) (ablation of Sec. 6.3)
//   block3d    4x4x4 cubes in raster order of the cubes, raster inside a cube (ablation of Sec. 6.3)
__device__ __forceinline__ uint32_t token_key(int64_t n, int order, int H, int W, int b, int b2) {
  const uint32_t w = uint32_t(n % W);
  const int64_t th = n / W;
  const uint32_t t = uint32_t(th / H), h = uint32_t(th % H);
  switch (order) {
    case DFS_ORDER_RASTER: return uint32_t(n);
    case DFS_ORDER_HILBERT2D: {
      uint32_t x[2] = {h, w};
      return (t << (2 * b2)) | hilbert_index<2>(x, b2);
    }
    case DFS_ORDER_BLOCK3D: {
      const uint32_t ch = uint32_t(H + 3) / 4, cw = uint32_t(W + 3) / 4;
      const uint32_t cube = ((t / 4) * ch + h / 4) * cw + w / 4;
      return cube * 64u + ((t % 4) * 4u + h % 4) * 4u + w % 4;
    }
    default: {
      uint32_t x[3] = {t, h, w};
      return hilbert_index<3>(x, b);
    }
  }
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void mark_cells_kernel(uint32_t* bitmap, int64_t N_v, int order, int H, int W, int b, int b2) {
  int64_t n = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (n >= N_v) return;
  const uint32_t key = token_key(n, order, H, W, b, b2);
  atomicOr(&bitmap[key >> 5], 1u << (key & 31));
}

constexpr int SCAN_T = 256;

// Inclusive scan of one value per thread across a 256-thread block (wave shuffles + LDS).
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* wave_tot /*[4]*/) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    uint32_t up = __shfl_up(v, off, 64);
    if (lane >= off) v += up;
  }
  if (lane == 63) wave_tot[wave] = v;
  __syncthreads();
  uint32_t base = 0;
  for (int i = 0; i < wave; ++i) base += wave_tot[i];
  __syncthreads();
  return v + base;
}

// chunk_sum[c] = number of occupied cells in words [c*256, c*256+256)
__global__ void __launch_bounds__(SCAN_T) chunk_count_kernel(const uint32_t* bitmap, size_t n_words, uint32_t* chunk_sum) {
  __shared__ uint32_t wt[4];
  size_t i = blockIdx.x * size_t(SCAN_T) + threadIdx.x;
  uint32_t v = i < n_words ? __popc(bitmap[i]) : 0u;
  uint32_t inc = block_inclusive_scan(v, wt);
  if (threadIdx.x == SCAN_T - 1) chunk_sum[blockIdx.x] = inc;
}

// In-place exclusive scan of chunk_sum[0..n) by one block, carrying across passes of 256.
__global__ void __launch_bounds__(SCAN_T) chunk_scan_kernel(uint32_t* chunk_sum, size_t n) {
  __shared__ uint32_t wt[4];
  __shared__ uint32_t carry_s;
  uint32_t carry = 0;
  for (size_t base = 0; base < n; base += SCAN_T) {
    size_t i = base + threadIdx.x;
    uint32_t v = i < n ? chunk_sum[i] : 0u;
    uint32_t inc = block_inclusive_scan(v, wt);
    if (i < n) chunk_sum[i] = carry + inc - v;
    if (threadIdx.x == SCAN_T - 1) carry_s = carry + inc;
    __syncthreads();
    carry = carry_s;
    __syncthreads();
  }
}

// word_prefix[i] = number of occupied cells in words [0, i)
__global__ void __launch_bounds__(SCAN_T) word_prefix_kernel(const uint32_t* bitmap, size_t n_words, const uint32_t* chunk_off,
                                                             uint32_t* word_prefix) {
  __shared__ uint32_t wt[4];
  size_t i = blockIdx.x * size_t(SCAN_T) + threadIdx.x;
  uint32_t v = i < n_words ? __popc(bitmap[i]) : 0u;
  uint32_t inc = block_inclusive_scan(v, wt);
  if (i < n_words) word_prefix[i] = chunk_off[blockIdx.x] + inc - v;
}

// Every video token writes itself at its rank; text tokens and pads are filled in beside them.
__global__ void emit_perm_kernel(const uint32_t* bitmap, const uint32_t* word_prefix, int64_t N_v, int n_text, int order, int H,
                                 int W, int b, int b2, int B, int M_v, int64_t N_pad, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid) {
  int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i < N_v) {
    const uint32_t key = token_key(i, order, H, W, b, b2);
    const uint32_t word = bitmap[key >> 5];
    const uint32_t rank = word_prefix[key >> 5] + __popc(word & ((1u << (key & 31)) - 1u));
    perm_pad[rank] = int32_t(i);
    inv[i] = int32_t(rank);
  }
  if (i < N_pad) {
    const int64_t text_base = int64_t(M_v) * B;
    if (i >= N_v && i < text_base) perm_pad[i] = -1;
    if (i >= text_base) {
      const int64_t j = i - text_base;
      if (j < n_text) { perm_pad[i] = int32_t(N_v + j); inv[N_v + j] = int32_t(i); }
      else perm_pad[i] = -1;
    }
    if (i % B == 0) {
      const int64_t blk = i / B;
      int64_t real = blk < M_v ? N_v - blk * B : int64_t(n_text) - (blk - M_v) * B;
      blk_valid[blk] = int32_t(real > B ? B : (real < 0 ? 0 : real));
    }
  }
}

static inline int bits_for(int extent) {
  int b = 1;
  while ((1 << b) < extent) ++b;
  return b;
}

// Number of key values an order can produce for a geometry (every token's key is below it).
static size_t key_space(const dfs_geom* g, const dfs_sizes& s, int order) {
  switch (order) {
    case DFS_ORDER_RASTER: return size_t(s.N_v);
    case DFS_ORDER_HILBERT2D: return size_t(g->T) << (2 * bits_for(g->H > g->W ? g->H : g->W));
    case DFS_ORDER_BLOCK3D: return size_t((g->T + 3) / 4) * ((g->H + 3) / 4) * ((g->W + 3) / 4) * 64;
    default: return size_t(1) << (3 * s.bits);
  }
}
static inline size_t bitmap_words(size_t cells) { return (cells + 31) / 32; }

static size_t ws_for_cells(size_t cells) {
  const size_t nw = bitmap_words(cells);
  const size_t chunks = (nw + SCAN_T - 1) / SCAN_T;
  return align256(nw * 4) * 2 + align256(chunks * 4);
}

size_t ws_hilbert(const dfs_geom* g, const dfs_sizes& s) {   // enough for every order
  size_t need = 0;
  for (int order = 0; order < 4; ++order) {
    const size_t w = ws_for_cells(key_space(g, s, order));
    need = w > need ? w : need;
  }
  return need;
}

int run_token_order(const dfs_geom* g, const dfs_sizes& s, int order, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid, void* ws,
                    hipStream_t st) {
  const size_t cells = key_space(g, s, order);
  if (cells > (size_t(1) << 31)) return fail(DFS_ESHAPE, "token order: key space of %zu cells is too large", cells);
  const size_t nw = bitmap_words(cells);
  const size_t chunks = (nw + SCAN_T - 1) / SCAN_T;
  uint32_t* bitmap = static_cast<uint32_t*>(ws);
  uint32_t* prefix = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + align256(nw * 4));
  uint32_t* chunk = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + 2 * align256(nw * 4));
  const int b2 = bits_for(g->H > g->W ? g->H : g->W);
  fill_u32_kernel<<<dim3(unsigned((nw + 255) / 256)), 256, 0, st>>>(bitmap, nw, 0u);
  mark_cells_kernel<<<dim3(unsigned((s.N_v + 255) / 256)), 256, 0, st>>>(bitmap, s.N_v, order, g->H, g->W, s.bits, b2);
  chunk_count_kernel<<<dim3(unsigned(chunks)), SCAN_T, 0, st>>>(bitmap, nw, chunk);
  chunk_scan_kernel<<<1, SCAN_T, 0, st>>>(chunk, chunks);
  word_prefix_kernel<<<dim3(unsigned(chunks)), SCAN_T, 0, st>>>(bitmap, nw, chunk, prefix);
  const int64_t span = s.N_pad > s.N_v ? s.N_pad : s.N_v;
  emit_perm_kernel<<<dim3(unsigned((span + 255) / 256)), 256, 0, st>>>(bitmap, prefix, s.N_v, g->n_text, order, g->H, g->W, s.bits, b2,
                                                                     g->B, s.M_v, s.N_pad, perm_pad, inv, blk_valid);
  return launch_status("dfs_token_order");
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_token_order(const dfs_geom* g, int order, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid, void* ws,
                               size_t ws_bytes, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (order < DFS_ORDER_HILBERT3D || order > DFS_ORDER_BLOCK3D) return fail(DFS_EINVAL, "dfs_token_order: unknown order %d", order);
  if (!perm_pad || !inv || !blk_valid) return fail(DFS_EINVAL, "dfs_token_order: NULL output");
  const size_t need = ws_hilbert(g, s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_token_order: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_token_order(g, s, order, perm_pad, inv, blk_valid, ws, as_stream(stream));
}

extern "C" int dfs_hilbert_perm(const dfs_geom* g, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid, void* ws, size_t ws_bytes,
                                void* stream) {
  return dfs_token_order(g, DFS_ORDER_HILBERT3D, perm_pad, inv, blk_valid, ws, ws_bytes, stream);
}
