// Hierarchical block scoring (paper Sec. 5.2; Algorithm 1 step 2; Eq. 2 and Eq. 8).
//
//   pool_kernel   : Q_hat, K_hat = mean over the real rows of each sub-block, an HBM stream.  The fp32
//                   means (Q_hat already times 1/sqrt(d)) are stored split into three bf16 terms
//                   x = hi + mid + lo, which together carry the 24 bits of the fp32 value.
//   score_kernel  : S_hat[u,v] = sum over the r x r sub-block pairs of softmax(Q_hat K_hat^T / sqrt(d)).
//                   The sub-block attention matrix A_hat is never stored: a work-group owns 128 query
//                   sub-blocks (32 per wave) and walks all key sub-blocks twice (first pass: row maximum
//                   and normaliser, second pass: normalised probabilities folded r x r), writing only the
//                   block scores.  The logits run on the bf16 matrix cores as six partial products
//                   hi.hi + hi.mid + mid.hi + hi.lo + lo.hi + mid.mid with fp32 accumulation: every
//                   bf16 product is exact in fp32 and the dropped terms are below 2^-23 of the result, so
//                   the logits are as accurate as an fp32 contraction at 2.7 times its speed (the mask
//                   decision that follows stays an fp32 one).
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
                                                   const int32_t* __restrict__ q_index, int64_t N_src, int64_t N_pad, int64_t N_v, int Bs,
                                                   int M_s, float q_scale) {
  constexpr int EPL = BF16 ? 8 : 4;           // elements per lane (16 bytes)
  constexpr int TPR = D / EPL;                // lanes per row
  constexpr int RPP = 64 / TPR;               // rows per pass
  const int lane = threadIdx.x & 63;
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= M_s) return;
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
  const bool gather = blockIdx.z == 0 && q_index != nullptr;
  const u32x4* base = reinterpret_cast<const u32x4*>(src) + (gather ? int64_t(head) * N_src * TPR : (int64_t(head) * N_pad + row0) * TPR) + c;
  for (int i = rg; i < cnt; i += RPP) {
    int64_t from = i;
    if (gather) {
      from = q_index[row0 + i];
      if (from < 0 || from >= N_src) continue;
    }
    const u32x4 v = __builtin_nontemporal_load(base + from * TPR);
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

// Running (max, sum of exp) of a softmax row; merge of two partial rows.
__device__ __forceinline__ void online_add(float& m, float& z, float x) {
  const float e = __expf(-fabsf(x - m));
  if (x > m) { z = z * e + 1.f; m = x; } else { z += e; }
}
__device__ __forceinline__ void online_merge(float& m, float& z, float m2, float z2) {
  const float mx = fmaxf(m, m2);
  if (mx == -INFINITY) { z = 0.f; return; }
  z = z * __expf(m - mx) + z2 * __expf(m2 - mx);
  m = mx;
}

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
score_kernel(const uint16_t* __restrict__ q_hat, const uint16_t* __restrict__ k_hat, float* __restrict__ score, int M_s, int M_v,
             int r, int n_live) {
  constexpr int RS = 3 * D;                   // elements of a centroid row (hi, mid, lo planes)
  constexpr int RSP = RS + 8;                 // LDS row stride: 16 bytes of skew keep the row-per-lane reads conflict-free
  constexpr int KS = D / 16;                  // product steps of 16 features
  constexpr int CPT = 32 * RS / 8 / 256;      // 16-byte chunks of a key tile per thread (6 at d=128)
  __shared__ __attribute__((aligned(16))) uint16_t s_k[32 * RSP];
  __shared__ float s_p[4][32][33];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  const int head = blockIdx.y;
  const int i0 = blockIdx.x * 128 + wave * 32;   // first query sub-block of this wave
  const uint16_t* qh = q_hat + int64_t(head) * M_s * RS;
  const uint16_t* kh = k_hat + int64_t(head) * M_s * RS;

  // Query centroids as the A operand: lane (n, half) holds row i0 + n, features 16 kk + 8 half .. + 7, three planes.
  bf16x8 aq[3][KS];
  {
    const int row = i0 + n;
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (row < M_s) v = *reinterpret_cast<const u32x4*>(qh + int64_t(row) * RS + p * D + 16 * kk + 8 * half);
        aq[p][kk] = __builtin_bit_cast(bf16x8, v);
      }
  }
  const int n_tiles = (n_live + 31) / 32;     // key sub-blocks at or beyond n_live are empty

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
  auto commit = [&]() {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<u32x4*>(&s_k[(c / (RS / 8)) * RSP + (c % (RS / 8)) * 8]) = stage[i];
    }
  };
  // logits of the 32 x 32 tile: c[i] = <q_hat[row 8 (i/4) + 4 half + i%4], k_hat[column n]>
  auto logit_tile = [&]() {
    // three accumulators, so that consecutive matrix instructions never wait for each other's result
    f32x16 sa = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 sb = sa, big = sa;
    const uint16_t* krow = &s_k[n * RSP + 8 * half];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(krow + 16 * kk));
      const bf16x8 bm = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(krow + D + 16 * kk));
      const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(krow + 2 * D + 16 * kk));
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[2][kk], bh, sa, 0, 0, 0);     // lo.hi
      sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[0][kk], bl, sb, 0, 0, 0);     // hi.lo
      big = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[0][kk], bh, big, 0, 0, 0);   // hi.hi
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[1][kk], bm, sa, 0, 0, 0);     // mid.mid
      sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[1][kk], bh, sb, 0, 0, 0);     // mid.hi
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[0][kk], bm, sa, 0, 0, 0);     // hi.mid
    }
    const f32x16 small = sa + sb;
    return big + small;
  };

  // pass 1: row maximum and normaliser.  Lane (n, half) holds rows 8 (i/4) + 4 half + i%4 of column n.
  float m[16], z[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { m[i] = -INFINITY; z[i] = 0.f; }
  fetch(0);
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();                          // every wave is done with the previous tile
    commit();
    __syncthreads();
    if (t + 1 < n_tiles) fetch(t + 1);
    const f32x16 c = logit_tile();
    if (t * 32 + n < n_live) {
#pragma unroll
      for (int i = 0; i < 16; ++i) online_add(m[i], z[i], c[i]);
    }
  }
#pragma unroll
  for (int off = 1; off < 32; off <<= 1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float m2 = __shfl_xor(m[i], off, 64), z2 = __shfl_xor(z[i], off, 64);
      online_merge(m[i], z[i], m2, z2);
    }
  }
  float rinv[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = i0 + 8 * (i / 4) + 4 * half + (i % 4);
    rinv[i] = (row < n_live && z[i] > 0.f) ? 1.0f / z[i] : 0.f;   // empty query sub-blocks score nothing
  }

  // pass 2: probabilities, folded r x r into block scores
  const int per = 32 / r;                     // blocks per tile edge
  const int u0 = i0 / r;
  float* out = score + int64_t(head) * M_v * M_v;
  const int n_tiles_all = (M_s + 31) / 32;
  fetch(0);
  for (int t = 0; t < n_tiles_all; ++t) {
    __syncthreads();
    commit();
    __syncthreads();
    if (t + 1 < n_tiles_all) fetch(t + 1);
    if (t < n_tiles) {
      const f32x16 c = logit_tile();
      const bool live = t * 32 + n < n_live;
#pragma unroll
      for (int i = 0; i < 16; ++i) s_p[wave][8 * (i / 4) + 4 * half + (i % 4)][n] = live ? __expf(c[i] - m[i]) * rinv[i] : 0.f;
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) s_p[wave][8 * (i / 4) + 4 * half + (i % 4)][n] = 0.f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // s_p[wave] is private to this wave: order its writes before its reads
    __builtin_amdgcn_wave_barrier();
    for (int o = lane; o < per * per; o += 64) {
      const int ur = o / per, vc = o % per;
      float acc = 0.f;
      for (int a = 0; a < r; ++a)
        for (int b = 0; b < r; ++b) acc += s_p[wave][ur * r + a][vc * r + b];
      const int u = u0 + ur, v = t * per + vc;
      if (u < M_v && v < M_v) out[int64_t(u) * M_v + v] = acc;
    }
    __builtin_amdgcn_wave_barrier();
  }
}

size_t ws_block_score(const dfs_geom* g, const dfs_sizes& s) {
  return 2 * align256(size_t(g->heads) * s.M_s * 3 * g->d * sizeof(uint16_t));
}

int run_block_score(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q_perm, const void* k_perm, float* score,
                    void* ws, const int32_t* q_index, hipStream_t st) {
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  const size_t half = align256(size_t(g->heads) * s.M_s * 3 * g->d * sizeof(uint16_t));
  uint16_t* q_hat = static_cast<uint16_t*>(ws);
  uint16_t* k_hat = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + half);
  dim3 pg(unsigned((s.M_s + 3) / 4), unsigned(g->heads), 2);
  const bool bf = dtype == DFS_BF16;
  const float scale = 1.0f / sqrtf(float(g->d));
#define POOL(BF, DD) pool_kernel<BF, DD><<<pg, 256, 0, st>>>(q_perm, k_perm, q_hat, k_hat, q_index, s.N, s.N_pad, s.N_v, g->Bs, s.M_s, scale)
  if (g->d == 64) { if (bf) POOL(true, 64); else POOL(false, 64); }
  else            { if (bf) POOL(true, 128); else POOL(false, 128); }
#undef POOL
  const int n_live = int((s.N_v + g->Bs - 1) / g->Bs);
  dim3 sg(unsigned((s.M_s + 127) / 128), unsigned(g->heads));
  if (g->d == 64) score_kernel<64><<<sg, 256, 0, st>>>(q_hat, k_hat, score, s.M_s, s.M_v, s.r, n_live);
  else score_kernel<128><<<sg, 256, 0, st>>>(q_hat, k_hat, score, s.M_s, s.M_v, s.r, n_live);
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
  const size_t need = ws_block_score(g, s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_block_score: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_block_score(g, s, dtype, q_perm, k_perm, score, ws, nullptr, as_stream(stream));
}

extern "C" int dfs_block_score_src(const dfs_geom* g, int dtype, const void* q, const int32_t* perm_pad, const void* k_perm,
                                   float* score, void* ws, size_t ws_bytes, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_BF16) return fail(DFS_EDTYPE, "dfs_block_score_src: bf16 tensors only");
  if (!q || !perm_pad || !k_perm || !score) return fail(DFS_EINVAL, "dfs_block_score_src: NULL argument");
  const size_t need = ws_block_score(g, s);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < need)
    return fail(DFS_EWORKSPACE, "dfs_block_score_src: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_block_score(g, s, dtype, q, k_perm, score, ws, perm_pad, as_stream(stream));
}
