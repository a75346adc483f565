// Token permutation by 3D Hilbert index (paper Sec. 5.1; Algorithm 1 step 1).
//
// Keys are ranked without a sort: every token sets the bit of its cell in a bitmap over the
// enclosing 2^b cube, a prefix sum over the bitmap words turns a cell into its rank among the
// occupied cells, and every token then writes itself at its rank.  Integer work only; run once
// per geometry.
#include "common.h"

namespace dfs {

// Hilbert index of cell (x0,x1,x2) in [0,2^b)^3: Butz curve in Skilling's transpose form.
// Level by level from the coarsest bit, a set bit of an axis reflects the lower bits of x0 and a
// clear bit exchanges the lower bits of x0 with that axis; a Gray decode across the axes follows;
// the three words are then read as b octal digits with x0 the high bit.
__device__ __forceinline__ uint32_t hilbert_index(uint32_t x0, uint32_t x1, uint32_t x2, int b) {
  uint32_t x[3] = {x0, x1, x2};
  for (uint32_t q = 1u << (b - 1); q > 1; q >>= 1) {
    const uint32_t low = q - 1;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
      if (x[a] & q) {
        x[0] ^= low;
      } else {
        const uint32_t swap = (x[0] ^ x[a]) & low;
        x[0] ^= swap;
        x[a] ^= swap;
      }
    }
  }
  x[1] ^= x[0];
  x[2] ^= x[1];
  uint32_t fix = 0;
  for (uint32_t q = 1u << (b - 1); q > 1; q >>= 1)
    if (x[2] & q) fix ^= q - 1;
  x[0] ^= fix; x[1] ^= fix; x[2] ^= fix;
  uint32_t key = 0;
  for (int j = b - 1; j >= 0; --j)
    key = (key << 3) | (((x[0] >> j) & 1u) << 2) | (((x[1] >> j) & 1u) << 1) | ((x[2] >> j) & 1u);
  return key;
}

__device__ __forceinline__ uint32_t token_key(int64_t n, int H, int W, int b) {
  const uint32_t w = uint32_t(n % W);
  const int64_t th = n / W;
  return hilbert_index(uint32_t(th / H), uint32_t(th % H), w, b);
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void mark_cells_kernel(uint32_t* bitmap, int64_t N_v, int H, int W, int b) {
  int64_t n = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (n >= N_v) return;
  const uint32_t key = token_key(n, H, W, b);
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
__global__ void emit_perm_kernel(const uint32_t* bitmap, const uint32_t* word_prefix, int64_t N_v, int n_text, int H, int W,
                                 int b, int B, int M_v, int64_t N_pad, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid) {
  int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i < N_v) {
    const uint32_t key = token_key(i, H, W, b);
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

static inline size_t bitmap_words(const dfs_sizes& s) {
  size_t cells = size_t(1) << (3 * s.bits);
  return cells < 32 ? 1 : cells / 32;
}

size_t ws_hilbert(const dfs_sizes& s) {
  size_t nw = bitmap_words(s);
  size_t chunks = (nw + SCAN_T - 1) / SCAN_T;
  return align256(nw * 4) * 2 + align256(chunks * 4);
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_hilbert_perm(const dfs_geom* g, int32_t* perm_pad, int32_t* inv, int32_t* blk_valid, void* ws,
                                size_t ws_bytes, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (!perm_pad || !inv || !blk_valid) return fail(DFS_EINVAL, "dfs_hilbert_perm: NULL output");
  const size_t need = ws_hilbert(s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_hilbert_perm: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  hipStream_t st = as_stream(stream);
  const size_t nw = bitmap_words(s);
  const size_t chunks = (nw + SCAN_T - 1) / SCAN_T;
  uint32_t* bitmap = static_cast<uint32_t*>(ws);
  uint32_t* prefix = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + align256(nw * 4));
  uint32_t* chunk = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + 2 * align256(nw * 4));
  fill_u32_kernel<<<dim3(unsigned((nw + 255) / 256)), 256, 0, st>>>(bitmap, nw, 0u);
  mark_cells_kernel<<<dim3(unsigned((s.N_v + 255) / 256)), 256, 0, st>>>(bitmap, s.N_v, g->H, g->W, s.bits);
  chunk_count_kernel<<<dim3(unsigned(chunks)), SCAN_T, 0, st>>>(bitmap, nw, chunk);
  chunk_scan_kernel<<<1, SCAN_T, 0, st>>>(chunk, chunks);
  word_prefix_kernel<<<dim3(unsigned(chunks)), SCAN_T, 0, st>>>(bitmap, nw, chunk, prefix);
  const int64_t span = s.N_pad > s.N_v ? s.N_pad : s.N_v;
  emit_perm_kernel<<<dim3(unsigned((span + 255) / 256)), 256, 0, st>>>(bitmap, prefix, s.N_v, g->n_text, g->H, g->W, s.bits,
                                                                     g->B, s.M_v, s.N_pad, perm_pad, inv, blk_valid);
  return launch_status("dfs_hilbert_perm");
}
