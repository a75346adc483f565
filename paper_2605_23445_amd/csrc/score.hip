// Hierarchical block scoring (paper Sec. 5.2; Algorithm 1 step 2; Eq. 2 and Eq. 8).
//
//   pool_kernel   : Q_hat, K_hat = mean over the real rows of each sub-block, an HBM stream.  The fp32
//                   means (Q_hat already times 1/sqrt(d)) are stored split into three bf16 terms
//                   x = hi + mid + lo, which together carry the 24 bits of the fp32 value.
//   score_lse_kernel / score_fold_kernel : S_hat[u,v] = sum over the r x r sub-block pairs of
//                   softmax(Q_hat K_hat^T / sqrt(d)).  The sub-block attention matrix A_hat is never stored.
//                   One pass over the contraction: per (query sub-block, key block) the base-2 log of the
//                   summed exponentials of the block's key sub-blocks (which needs no row reference) and per
//                   query sub-block the row log-sum-exp; a second, memory-bound kernel turns these into
//                   probabilities and folds the r query sub-blocks of a query block.  The logits run on the
//                   bf16 matrix cores as six partial products hi.hi + hi.mid + mid.hi + hi.lo + lo.hi +
//                   mid.mid with fp32 accumulation: every bf16 product is exact in fp32 and the dropped terms
//                   are below 2^-23 of the result, so the logits are as accurate as an fp32 contraction at
//                   several times its speed (the mask decision that follows stays an fp32 one).
#include "common.h"

namespace dfs {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------ pooling

// x -> (hi, mid, lo) with hi = bf16(x), mid = bf16(x - hi), lo = bf16(x - hi - mid); the subtractions are exact.
__device__ __forceinline__ void split3(float x, uint16_t& hi, uint16_t& mid, uint16_t& lo) {
  hi = f32_to_bf16(x);
  const float r1 = x - bf16_to_f32(hi);
  mid = f32_to_bf16(r1);
  const float r2 = r1 - bf16_to_f32(mid);
  lo = f32_to_bf16(r2);
}

// One wave per sub-block.  Lanes of a row sit side by side (16 bytes each); several rows are in
// flight per load; partial sums of the row groups are folded with cross-lane exchanges.
// Output row layout: [3][D] bf16 (hi, mid, lo planes).
template <bool BF16, int D>
__global__ void __launch_bounds__(256) pool_kernel(const void* __restrict__ q_perm, const void* __restrict__ k_perm,
                                                   uint16_t* __restrict__ q_hat, uint16_t* __restrict__ k_hat,
                                                   const int32_t* __restrict__ q_index, void* __restrict__ k_out, int64_t N_src,
                                                   int64_t N_pad, int64_t N_v, int Bs, int M_s, float q_scale) {
  constexpr int EPL = BF16 ? 8 : 4;           // elements per lane (16 bytes)
  constexpr int TPR = D / EPL;                // lanes per row
  constexpr int RPP = 64 / TPR;               // rows per pass
  const int lane = threadIdx.x & 63;
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  // With k_out the key rows come in source order too: they are gathered through the permutation, pooled, and
  // written out in the reordered layout on the way (pads as zeros), which spares the reorder pass of K.  The
  // sub-blocks behind the video segment (text rows) are then copied only.
  const bool k_copy = blockIdx.z == 1 && k_out != nullptr;
  if (s >= M_s && !(k_copy && int64_t(s) * Bs < N_pad)) return;
  const int head = blockIdx.y;
  const void* src = blockIdx.z == 0 ? q_perm : k_perm;
  uint16_t* dst = blockIdx.z == 0 ? q_hat : k_hat;
  const int c = lane % TPR, rg = lane / TPR;
  const int64_t row0 = int64_t(s) * Bs;
  int64_t left = N_v - row0;
  const int cnt = left <= 0 ? 0 : (left < Bs ? int(left) : Bs);
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  // With q_index (the permutation) the query rows are gathered from the tensor in source order, which spares
  // the reorder pass of Q.
  const bool gather = q_index != nullptr && (blockIdx.z == 0 || k_copy);
  const u32x4* base = reinterpret_cast<const u32x4*>(src) + (gather ? int64_t(head) * N_src * TPR : (int64_t(head) * N_pad + row0) * TPR) + c;
  u32x4* copy = k_copy ? reinterpret_cast<u32x4*>(k_out) + (int64_t(head) * N_pad + row0) * TPR + c : nullptr;
  const int rows = k_copy ? Bs : cnt;         // a copy covers the pad rows of the sub-block as well
  for (int i = rg; i < rows; i += RPP) {
    int64_t from = i;
    bool real = true;
    if (gather) {
      from = q_index[row0 + i];
      real = from >= 0 && from < N_src;
    }
    if (!real && !k_copy) continue;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (real) v = __builtin_nontemporal_load(base + from * TPR);
    if (k_copy) __builtin_nontemporal_store(v, copy + int64_t(i) * TPR);
    if (!real || i >= cnt) continue;
    if (BF16) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += __uint_as_float(v[e] << 16);
        acc[2 * e + 1] += __uint_as_float(v[e] & 0xFFFF0000u);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] += __uint_as_float(v[e]);
    }
  }
  if (s >= M_s) return;                        // copied only
#pragma unroll
  for (int off = TPR; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
  }
  if (rg == 0) {
    const float inv = cnt > 0 ? (blockIdx.z == 0 ? q_scale : 1.0f) / float(cnt) : 0.f;
    uint16_t* o = dst + (int64_t(head) * M_s + s) * (3 * D) + c * EPL;
    uint16_t hi[EPL], mid[EPL], lo[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) split3(acc[e] * inv, hi[e], mid[e], lo[e]);
#pragma unroll
    for (int e = 0; e < EPL; e += 2) {
      *reinterpret_cast<uint32_t*>(o + e) = uint32_t(hi[e]) | (uint32_t(hi[e + 1]) << 16);
      *reinterpret_cast<uint32_t*>(o + D + e) = uint32_t(mid[e]) | (uint32_t(mid[e + 1]) << 16);
      *reinterpret_cast<uint32_t*>(o + 2 * D + e) = uint32_t(lo[e]) | (uint32_t(lo[e + 1]) << 16);
    }
  }
}

// ------------------------------------------------------------------------------------ scoring

constexpr float LSE_START = -1.0e30f;          // finite stand-in for "nothing seen yet" (keeps differences finite)

// Running base-2 log-sum-exp (reference m, sum z of 2^(x - m)): add one term, merge two partial sums.
__device__ __forceinline__ void lse_add(float& m, float& z, float x) {
  const float mn = fmaxf(m, x);
  z = z * __builtin_amdgcn_exp2f(m - mn) + __builtin_amdgcn_exp2f(x - mn);
  m = mn;
}
__device__ __forceinline__ void lse_merge(float& m, float& z, float m2, float z2) {
  const float mn = fmaxf(m, m2);
  z = z * __builtin_amdgcn_exp2f(m - mn) + z2 * __builtin_amdgcn_exp2f(m2 - mn);
  m = mn;
}

// Pass 1 (the contraction, once).  A work-group owns 128 query sub-blocks (32 per wave) and one of KSPLIT
// ranges of key tiles (32 key sub-blocks each).  The logits are computed transposed, keys along the rows of
// the matrix instruction's result, so that a lane holds, for ONE query sub-block (its column), runs of four
// consecutive key sub-blocks: the R key sub-blocks of a key block fold inside the lane (R = 8: plus one
// exchange between the two lane halves).  Per (query sub-block i, key block v) it stores
//   T[v][i] = log2 sum over the key sub-blocks j of v of 2^logit(i, j)          (logits already in base 2)
// which needs no row reference, and per query sub-block the log-sum-exp over its key range.  Pass 2 turns
// T into probabilities and folds the R query sub-blocks of a query block.
template <int D, int R>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
score_lse_kernel(const uint16_t* __restrict__ q_hat, const uint16_t* __restrict__ k_hat, float* __restrict__ tt,
                 float* __restrict__ lse, int M_s, int M_v, int n_live, int tiles_per_split, int ksplit) {
  constexpr int RS = 3 * D;                   // elements of a centroid row (hi, mid, lo planes)
  constexpr int RSP = RS + 8;                 // LDS row stride: 16 bytes of skew keep the row-per-lane reads conflict-free
  constexpr int KS = D / 16;                  // product steps of 16 features
  constexpr int CPT = 32 * RS / 8 / 256;      // 16-byte chunks of a key tile per thread (6 at d=128)
  constexpr int G = R < 4 ? R : 4;            // key sub-blocks of one key block that sit in consecutive registers
  __shared__ __attribute__((aligned(16))) uint16_t s_k[2][32 * RSP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  const int head = blockIdx.y;
  const int split = blockIdx.x % ksplit;
  const int i0 = (blockIdx.x / ksplit) * 128 + wave * 32;   // first query sub-block of this wave
  const uint16_t* qh = q_hat + int64_t(head) * M_s * RS;
  const uint16_t* kh = k_hat + int64_t(head) * M_s * RS;

  // Query centroids as the B operand: lane (n, half) holds row i0 + n, features 16 kk + 8 half .. + 7, three planes.
  bf16x8 bq[3][KS];
  {
    const int row = i0 + n;
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (row < M_s) v = *reinterpret_cast<const u32x4*>(qh + int64_t(row) * RS + p * D + 16 * kk + 8 * half);
        bq[p][kk] = __builtin_bit_cast(bf16x8, v);
      }
  }
  const int n_tiles = (n_live + 31) / 32;     // key sub-blocks at or beyond n_live are empty
  const int t_begin = split * tiles_per_split;
  const int t_end = t_begin + tiles_per_split < n_tiles ? t_begin + tiles_per_split : n_tiles;

  // key tile t (32 centroid rows, contiguous in memory) -> registers -> LDS
  u32x4 stage[CPT];
  auto fetch = [&](int t) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * 256;
      const int row = t * 32 + c / (RS / 8);
      stage[i] = u32x4{0u, 0u, 0u, 0u};
      if (row < M_s) stage[i] = *reinterpret_cast<const u32x4*>(kh + int64_t(t) * 32 * RS + int64_t(c) * 8);
    }
  };
  auto commit = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<u32x4*>(&s_k[buf][(c / (RS / 8)) * RSP + (c % (RS / 8)) * 8]) = stage[i];
    }
  };
  // transposed logits of the 32 x 32 tile: c[i] = <k_hat[row 8 (i/4) + 4 half + i%4 of the tile], q_hat[i0 + n]>
  auto logit_tile = [&](int buf) {
    // three accumulators, so that consecutive matrix instructions never wait for each other's result
    f32x16 sa = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 sb = sa, big = sa;
    const uint16_t* krow = &s_k[buf][n * RSP + 8 * half];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(krow + 16 * kk));
      const bf16x8 am = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(krow + D + 16 * kk));
      const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(krow + 2 * D + 16 * kk));
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bq[2][kk], sa, 0, 0, 0);     // hi.lo
      sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bq[0][kk], sb, 0, 0, 0);     // lo.hi
      big = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bq[0][kk], big, 0, 0, 0);   // hi.hi
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bq[1][kk], sa, 0, 0, 0);     // mid.mid
      sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bq[1][kk], sb, 0, 0, 0);     // hi.mid
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bq[0][kk], sa, 0, 0, 0);     // mid.hi
    }
    const f32x16 small = sa + sb;
    return big + small;
  };

  float m_row = LSE_START, z_row = 0.f;       // this lane's share of the row log-sum-exp of query sub-block i0 + n
  const int q_row = i0 + n;
  float* tt_h = tt + int64_t(head) * M_v * M_s;
  if (t_begin < t_end) {
    fetch(t_begin);
    commit(0);
    __syncthreads();
    for (int t = t_begin; t < t_end; ++t) {
      const int buf = (t - t_begin) & 1;
      if (t + 1 < t_end) fetch(t + 1);
      f32x16 c = logit_tile(buf);
      if (t + 1 < t_end) commit(buf ^ 1);     // the other buffer was last read before the previous barrier
      if (t * 32 + 32 > n_live) {             // ragged end: key sub-blocks without rows count for nothing
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (t * 32 + 8 * (i / 4) + 4 * half + (i % 4) >= n_live) c[i] = -INFINITY;
      }
      // fold the key sub-blocks of each key block: groups of G consecutive registers
#pragma unroll
      for (int gi = 0; gi < 16 / G; ++gi) {
        float mg = c[gi * G];
#pragma unroll
        for (int e = 1; e < G; ++e) mg = fmaxf(mg, c[gi * G + e]);
        float sg = 0.f;
        const float ref = mg == -INFINITY ? 0.f : mg;
#pragma unroll
        for (int e = 0; e < G; ++e) sg += __builtin_amdgcn_exp2f(c[gi * G + e] - ref);
        float tv = mg == -INFINITY ? -INFINITY : mg + __builtin_amdgcn_logf(sg);
        // key sub-block of the group's first register: 8 (first / 4) + 4 half + first % 4
        const int first = gi * G;
        const int ks = t * 32 + 8 * (first / 4) + 4 * half + (first % 4);
        if (R == 8) {                          // the other half of the block sits in lane ^ 32
          const float other = __shfl_xor(tv, 32, 64);
          float m2 = fmaxf(tv, other);
          tv = m2 == -INFINITY ? -INFINITY
                               : m2 + __builtin_amdgcn_logf(__builtin_amdgcn_exp2f(tv - m2) + __builtin_amdgcn_exp2f(other - m2));
        }
        const int v = ks / R;
        if ((R != 8 || half == 0) && v < M_v && q_row < M_s) tt_h[int64_t(v) * M_s + q_row] = tv;
        if (R != 8 || half == 0) lse_add(m_row, z_row, tv);
      }
      __syncthreads();                        // tile t has been read by every wave; tile t + 1 is in LDS
    }
  }
  // the two lane halves of a column hold different key blocks of the same query sub-block
  {
    const float m2 = __shfl_xor(m_row, 32, 64), z2 = __shfl_xor(z_row, 32, 64);
    lse_merge(m_row, z_row, m2, z2);
  }
  if (half == 0 && q_row < M_s)
    lse[(int64_t(head) * ksplit + split) * M_s + q_row] = z_row > 0.f ? m_row + __builtin_amdgcn_logf(z_row) : -INFINITY;
}

// Pass 2: S_hat[u][v] = sum over the R query sub-blocks i of u of 2^(T[v][i] - lse(i)), lse(i) merged over the
// key ranges.  A work-group handles 32 query blocks x 32 key blocks; T is read along i (contiguous), the
// scores are written along v (contiguous), the transposition goes through LDS.
template <int R>
__global__ void __launch_bounds__(256) score_fold_kernel(const float* __restrict__ tt, const float* __restrict__ lse,
                                                         float* __restrict__ score, int M_s, int M_v, int n_live, int ksplit) {
  __shared__ float s_t[32][33];
  const int head = blockIdx.z, u0 = blockIdx.x * 32, v0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 x 8
  const float* tt_h = tt + int64_t(head) * M_v * M_s;
  const float* lse_h = lse + int64_t(head) * ksplit * M_s;
  // row log-sum-exp of the R sub-blocks of query block u0 + tx
  float l[R];
#pragma unroll
  for (int a = 0; a < R; ++a) {
    const int i = (u0 + tx) * R + a;
    float m = LSE_START, z = 0.f;
    if (u0 + tx < M_v && i < n_live) {
      for (int sp = 0; sp < ksplit; ++sp) lse_add(m, z, lse_h[int64_t(sp) * M_s + i]);
    }
    l[a] = z > 0.f ? m + __builtin_amdgcn_logf(z) : INFINITY;       // +inf: an empty query sub-block scores nothing
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int v = v0 + ty + 8 * k;
    float acc = 0.f;
    if (v < M_v && u0 + tx < M_v) {
      const float* row = tt_h + int64_t(v) * M_s + int64_t(u0 + tx) * R;
#pragma unroll
      for (int a = 0; a < R; ++a) acc += __builtin_amdgcn_exp2f(row[a] - l[a]);
    }
    s_t[ty + 8 * k][tx] = acc;                                       // [v][u]
  }
  __syncthreads();
  float* out = score + int64_t(head) * M_v * M_v;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int u = u0 + ty + 8 * k, v = v0 + tx;
    if (u < M_v && v < M_v) out[int64_t(u) * M_v + v] = s_t[tx][ty + 8 * k];
  }
}

// Workspace: Q_hat, K_hat (three bf16 planes each), T [heads][M_v][M_s] fp32, row log-sum-exp
// [heads][KSPLIT_MAX][M_s] fp32.
constexpr int KSPLIT_MAX = 4;
static size_t ws_hat_bytes(const dfs_geom* g, const dfs_sizes& s) { return align256(size_t(g->heads) * s.M_s * 3 * g->d * sizeof(uint16_t)); }
static size_t ws_tt_bytes(const dfs_geom* g, const dfs_sizes& s) { return align256(size_t(g->heads) * s.M_v * s.M_s * sizeof(float)); }
static size_t ws_lse_bytes(const dfs_geom* g, const dfs_sizes& s) { return align256(size_t(g->heads) * KSPLIT_MAX * s.M_s * sizeof(float)); }
size_t ws_block_score(const dfs_geom* g, const dfs_sizes& s) {
  return 2 * ws_hat_bytes(g, s) + ws_tt_bytes(g, s) + ws_lse_bytes(g, s);
}

// Key ranges per query group: the split that wastes the least of the last round of work-groups
// (512 work-groups of 4 waves are resident on the chip at two waves per SIMD).
static int choose_ksplit(int64_t groups_times_heads, int n_tiles) {
  int best = 1;
  double best_cost = 1e300;
  for (int k = 1; k <= KSPLIT_MAX; ++k) {
    const int per = (n_tiles + k - 1) / k;
    const int64_t wgs = groups_times_heads * k;
    const int64_t rounds = (wgs + 511) / 512;
    const double cost = double(rounds) * (per + 2);       // +2: prologue / epilogue of a work-group, in tile units
    if (cost < best_cost - 1e-9) { best_cost = cost; best = k; }
  }
  return best;
}

template <int D, int R>
static void launch_score(const dfs_geom* g, const dfs_sizes& s, const uint16_t* q_hat, const uint16_t* k_hat, float* tt, float* lse,
                         float* score, int n_live, hipStream_t st) {
  const int groups = (s.M_s + 127) / 128, n_tiles = (n_live + 31) / 32;
  const int ksplit = choose_ksplit(int64_t(groups) * g->heads, n_tiles);
  const int per = (n_tiles + ksplit - 1) / ksplit;
  score_lse_kernel<D, R><<<dim3(unsigned(groups * ksplit), unsigned(g->heads)), 256, 0, st>>>(q_hat, k_hat, tt, lse, s.M_s, s.M_v, n_live,
                                                                                              per, ksplit);
  const unsigned tb = unsigned((s.M_v + 31) / 32);
  score_fold_kernel<R><<<dim3(tb, tb, unsigned(g->heads)), 256, 0, st>>>(tt, lse, score, s.M_s, s.M_v, n_live, ksplit);
}

int run_block_score(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q_perm, const void* k_perm, float* score,
                    void* ws, const int32_t* q_index, void* k_out, hipStream_t st) {
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  if ((s.M_v + 31) / 32 > 65535) return fail(DFS_ESHAPE, "M_v=%d is too large for the scoring grid", s.M_v);
  char* base = static_cast<char*>(ws);
  uint16_t* q_hat = reinterpret_cast<uint16_t*>(base);
  uint16_t* k_hat = reinterpret_cast<uint16_t*>(base + ws_hat_bytes(g, s));
  float* tt = reinterpret_cast<float*>(base + 2 * ws_hat_bytes(g, s));
  float* lse = reinterpret_cast<float*>(base + 2 * ws_hat_bytes(g, s) + ws_tt_bytes(g, s));
  const int64_t pool_subs = k_out ? s.N_pad / g->Bs : s.M_s;   // with k_out the text blocks are copied as well
  dim3 pg(unsigned((pool_subs + 3) / 4), unsigned(g->heads), 2);
  const bool bf = dtype == DFS_BF16;
  // 1/sqrt(d) of Eq. 2 and the change to base 2 go into Q_hat, so that the logits come out of the contraction in base 2
  const float scale = 1.4426950408889634f / sqrtf(float(g->d));
#define POOL(BF, DD) pool_kernel<BF, DD><<<pg, 256, 0, st>>>(q_perm, k_perm, q_hat, k_hat, q_index, k_out, s.N, s.N_pad, s.N_v, g->Bs, s.M_s, scale)
  if (g->d == 64) { if (bf) POOL(true, 64); else POOL(false, 64); }
  else            { if (bf) POOL(true, 128); else POOL(false, 128); }
#undef POOL
  const int n_live = int((s.N_v + g->Bs - 1) / g->Bs);
#define SCORE(DD, RR) launch_score<DD, RR>(g, s, q_hat, k_hat, tt, lse, score, n_live, st)
#define SCORE_R(DD)                                                                 \
  switch (s.r) {                                                                    \
    case 1: SCORE(DD, 1); break;                                                    \
    case 2: SCORE(DD, 2); break;                                                    \
    case 4: SCORE(DD, 4); break;                                                    \
    case 8: SCORE(DD, 8); break;                                                    \
    default: return fail(DFS_ESHAPE, "B/Bs=%d is not 1, 2, 4 or 8", s.r);           \
  }
  if (g->d == 64) { SCORE_R(64) } else { SCORE_R(128) }
#undef SCORE_R
#undef SCORE
  return launch_status("dfs_block_score");
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_block_score(const dfs_geom* g, int dtype, const void* q_perm, const void* k_perm, float* score, void* ws,
                               size_t ws_bytes, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_F32 && dtype != DFS_BF16) return fail(DFS_EDTYPE, "dtype %d is not DFS_F32 or DFS_BF16", dtype);
  if (!q_perm || !k_perm || !score) return fail(DFS_EINVAL, "dfs_block_score: NULL argument");
  if (misaligned(16, {q_perm, k_perm}) || misaligned(4, {score})) return fail(DFS_EINVAL, "dfs_block_score: tensors must be 16-byte aligned, the score array 4-byte aligned");
  const size_t need = ws_block_score(g, s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_block_score: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_block_score(g, s, dtype, q_perm, k_perm, score, ws, nullptr, nullptr, as_stream(stream));
}

extern "C" int dfs_block_score_src(const dfs_geom* g, int dtype, const void* q, const int32_t* perm_pad, const void* k_perm,
                                   float* score, void* ws, size_t ws_bytes, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_BF16) return fail(DFS_EDTYPE, "dfs_block_score_src: bf16 tensors only");
  if (!q || !perm_pad || !k_perm || !score) return fail(DFS_EINVAL, "dfs_block_score_src: NULL argument");
  if (misaligned(16, {q, k_perm}) || misaligned(4, {perm_pad, score}))
    return fail(DFS_EINVAL, "dfs_block_score_src: tensors must be 16-byte aligned, index and score arrays 4-byte aligned");
  const size_t need = ws_block_score(g, s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_block_score_src: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_block_score(g, s, dtype, q, k_perm, score, ws, perm_pad, nullptr, as_stream(stream));
}

extern "C" int dfs_block_score_fused(const dfs_geom* g, int dtype, const void* q, const void* k, const int32_t* perm_pad,
                                     void* k_perm, float* score, void* ws, size_t ws_bytes, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_BF16) return fail(DFS_EDTYPE, "dfs_block_score_fused: bf16 tensors only");
  if (!q || !k || !perm_pad || !k_perm || !score) return fail(DFS_EINVAL, "dfs_block_score_fused: NULL argument");
  if (misaligned(16, {q, k, k_perm}) || misaligned(4, {perm_pad, score}))
    return fail(DFS_EINVAL, "dfs_block_score_fused: tensors must be 16-byte aligned, index and score arrays 4-byte aligned");
  if (k == k_perm) return fail(DFS_EINVAL, "dfs_block_score_fused: k_perm must not alias k");
  const size_t need = ws_block_score(g, s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_block_score_fused: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_block_score(g, s, dtype, q, k, score, ws, perm_pad, k_perm, as_stream(stream));
}
