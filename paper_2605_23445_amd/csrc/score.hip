// Hierarchical block scoring (paper Sec. 5.2; Algorithm 1 step 2; Eq. 2 and Eq. 8).
//
//   pool_kernel   : Q_hat, K_hat = mean over the real rows of each sub-block (fp32), an HBM stream.
//   score_kernel  : S_hat[u,v] = sum over the r x r sub-block pairs of softmax(Q_hat K_hat^T / sqrt(d)).
//                   The sub-block attention matrix A_hat is never stored: a work-group owns 32
//                   query sub-blocks, runs over all key sub-blocks twice with fp32 matrix-core
//                   products (first pass: row maximum and normaliser, second pass: normalised
//                   probabilities folded r x r) and writes only the block scores.
#include "common.h"

namespace dfs {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------ pooling

// One wave per sub-block.  Lanes of a row sit side by side (16 bytes each); several rows are in
// flight per load; partial sums of the row groups are folded with cross-lane exchanges.
template <bool BF16, int D>
__global__ void __launch_bounds__(256) pool_kernel(const void* __restrict__ q_perm, const void* __restrict__ k_perm,
                                                   float* __restrict__ q_hat, float* __restrict__ k_hat, int64_t N_pad,
                                                   int64_t N_v, int Bs, int M_s) {
  constexpr int EPL = BF16 ? 8 : 4;           // elements per lane (16 bytes)
  constexpr int TPR = D / EPL;                // lanes per row
  constexpr int RPP = 64 / TPR;               // rows per pass
  const int lane = threadIdx.x & 63;
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= M_s) return;
  const int head = blockIdx.y;
  const void* src = blockIdx.z == 0 ? q_perm : k_perm;
  float* dst = blockIdx.z == 0 ? q_hat : k_hat;
  const int c = lane % TPR, rg = lane / TPR;
  const int64_t row0 = int64_t(s) * Bs;
  int64_t left = N_v - row0;
  const int cnt = left <= 0 ? 0 : (left < Bs ? int(left) : Bs);
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  const u32x4* base = reinterpret_cast<const u32x4*>(src) + (int64_t(head) * N_pad + row0) * TPR + c;
  for (int i = rg; i < cnt; i += RPP) {
    const u32x4 v = __builtin_nontemporal_load(base + int64_t(i) * TPR);
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
    const float inv = cnt > 0 ? 1.0f / float(cnt) : 0.f;
    float* o = dst + (int64_t(head) * M_s + s) * D + c * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      f32x4 w = {acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv};
      *reinterpret_cast<f32x4*>(o + e) = w;
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

// logits of one 32 x 32 tile: rows = the work-group's query sub-blocks (held in `aq`), columns =
// key sub-blocks col0 .. col0+31.  Feature index of product step (kk, half) is half*D/2 + kk for
// both operands, so every lane reads D/2 consecutive floats of its key row.
template <int D>
__device__ __forceinline__ f32x16 logit_tile(const float (&aq)[D / 2], const float* __restrict__ k_hat_head, int col, int M_s,
                                             int half) {
  float bk[D / 2];
  if (col < M_s) {
    const f32x4* p = reinterpret_cast<const f32x4*>(k_hat_head + int64_t(col) * D + half * (D / 2));
#pragma unroll
    for (int j = 0; j < D / 8; ++j) {
      const f32x4 v = p[j];
      bk[4 * j] = v[0]; bk[4 * j + 1] = v[1]; bk[4 * j + 2] = v[2]; bk[4 * j + 3] = v[3];
    }
  } else {
#pragma unroll
    for (int j = 0; j < D / 2; ++j) bk[j] = 0.f;
  }
  f32x16 c = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < D / 2; ++kk) c = __builtin_amdgcn_mfma_f32_32x32x2f32(aq[kk], bk[kk], c, 0, 0, 0);
  return c;
}

template <int D>
__global__ void __launch_bounds__(256) score_kernel(const float* __restrict__ q_hat, const float* __restrict__ k_hat,
                                                    float* __restrict__ score, int M_s, int M_v, int r, int n_live,
                                                    float scale) {
  __shared__ float s_m[4][32], s_z[4][32];
  __shared__ float s_row_m[32], s_row_inv[32];
  __shared__ float s_p[4][32][33];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col_l = lane & 31, half = lane >> 5;
  const int head = blockIdx.y;
  const int i0 = blockIdx.x * 32;
  const float* qh = q_hat + int64_t(head) * M_s * D;
  const float* kh = k_hat + int64_t(head) * M_s * D;

  float aq[D / 2];
  {
    const int row = i0 + col_l;
    if (row < M_s) {
      const f32x4* p = reinterpret_cast<const f32x4*>(qh + int64_t(row) * D + half * (D / 2));
#pragma unroll
      for (int j = 0; j < D / 8; ++j) {
        const f32x4 v = p[j];
        aq[4 * j] = v[0] * scale; aq[4 * j + 1] = v[1] * scale; aq[4 * j + 2] = v[2] * scale; aq[4 * j + 3] = v[3] * scale;
      }
    } else {
#pragma unroll
      for (int j = 0; j < D / 2; ++j) aq[j] = 0.f;
    }
  }
  const int n_tiles = (n_live + 31) / 32;    // key sub-blocks at or beyond n_live are empty

  // pass 1: row maximum and normaliser.  Lane (col_l, half) holds rows 8*(i/4) + 4*half + i%4.
  float m[16], z[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { m[i] = -INFINITY; z[i] = 0.f; }
  for (int t = wave; t < n_tiles; t += 4) {
    const int col = t * 32 + col_l;
    const f32x16 c = logit_tile<D>(aq, kh, col, M_s, half);
    if (col < n_live) {
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
  if (col_l == 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = 8 * (i / 4) + 4 * half + (i % 4);
      s_m[wave][row] = m[i];
      s_z[wave][row] = z[i];
    }
  }
  __syncthreads();
  if (threadIdx.x < 32) {
    float mm = s_m[0][threadIdx.x], zz = s_z[0][threadIdx.x];
    for (int w = 1; w < 4; ++w) online_merge(mm, zz, s_m[w][threadIdx.x], s_z[w][threadIdx.x]);
    const int row = i0 + threadIdx.x;
    s_row_m[threadIdx.x] = mm;
    s_row_inv[threadIdx.x] = (row < n_live && zz > 0.f) ? 1.0f / zz : 0.f;   // empty query sub-blocks score nothing
  }
  __syncthreads();
  float rm[16], rinv[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = 8 * (i / 4) + 4 * half + (i % 4);
    rm[i] = s_row_m[row];
    rinv[i] = s_row_inv[row];
  }

  // pass 2: probabilities, folded r x r into block scores
  const int per = 32 / r;                    // blocks per tile edge
  const int u0 = i0 / r;
  float* out = score + int64_t(head) * M_v * M_v;
  const int n_tiles_all = (M_s + 31) / 32;
  for (int tb = 0; tb < n_tiles_all; tb += 4) {   // trip count is the same for all four waves
    const int t = tb + wave;
    const int col = t * 32 + col_l;
    if (t < n_tiles) {
      const f32x16 c = logit_tile<D>(aq, kh, col, M_s, half);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i / 4) + 4 * half + (i % 4);
        s_p[wave][row][col_l] = col < n_live ? __expf(c[i] - rm[i]) * rinv[i] : 0.f;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) s_p[wave][8 * (i / 4) + 4 * half + (i % 4)][col_l] = 0.f;
    }
    __syncthreads();
    if (t < n_tiles_all) {
      for (int o = lane; o < per * per; o += 64) {
        const int ur = o / per, vc = o % per;
        float acc = 0.f;
        for (int a = 0; a < r; ++a)
          for (int b = 0; b < r; ++b) acc += s_p[wave][ur * r + a][vc * r + b];
        const int u = u0 + ur, v = t * per + vc;
        if (u < M_v && v < M_v) out[int64_t(u) * M_v + v] = acc;
      }
    }
    __syncthreads();
  }
}

size_t ws_block_score(const dfs_geom* g, const dfs_sizes& s) {
  return 2 * align256(size_t(g->heads) * s.M_s * g->d * sizeof(float));
}

int run_block_score(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q_perm, const void* k_perm, float* score,
                    void* ws, hipStream_t st) {
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  const size_t half = align256(size_t(g->heads) * s.M_s * g->d * sizeof(float));
  float* q_hat = static_cast<float*>(ws);
  float* k_hat = reinterpret_cast<float*>(static_cast<char*>(ws) + half);
  dim3 pg(unsigned((s.M_s + 3) / 4), unsigned(g->heads), 2);
  const bool bf = dtype == DFS_BF16;
#define POOL(BF, DD) pool_kernel<BF, DD><<<pg, 256, 0, st>>>(q_perm, k_perm, q_hat, k_hat, s.N_pad, s.N_v, g->Bs, s.M_s)
  if (g->d == 64) { if (bf) POOL(true, 64); else POOL(false, 64); }
  else            { if (bf) POOL(true, 128); else POOL(false, 128); }
#undef POOL
  const int n_live = int((s.N_v + g->Bs - 1) / g->Bs);
  const float scale = 1.0f / sqrtf(float(g->d));
  dim3 sg(unsigned((s.M_s + 31) / 32), unsigned(g->heads));
  if (g->d == 64) score_kernel<64><<<sg, 256, 0, st>>>(q_hat, k_hat, score, s.M_s, s.M_v, s.r, n_live, scale);
  else score_kernel<128><<<sg, 256, 0, st>>>(q_hat, k_hat, score, s.M_s, s.M_v, s.r, n_live, scale);
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
  return run_block_score(g, s, dtype, q_perm, k_perm, score, ws, as_stream(stream));
}
