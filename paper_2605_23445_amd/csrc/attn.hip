// Block-sparse attention forward over the reordered sequence (paper Algorithm 1 step 3: Eq. 1
// restricted to the kept block pairs, softmax normalised over the kept keys).
//
// bf16 kernel (the hot one).  A work-group owns one query block of one head; each of its waves
// owns 32 query rows.  Key/value blocks named by kv_idx stream through LDS in tiles of 64 rows.
// Per tile a wave forms S^T = K Q^T on the matrix cores (32x32x16 bf16), so that every lane holds
// logits of ONE query row: the online-softmax maximum, normaliser and rescale factor are per-lane
// scalars and need a single exchange between lane l and l^32.  The probabilities, still in
// registers, are already laid out as the B operand of O^T += V^T P^T; the V^T operand comes out of
// LDS through the transposing LDS read, so V is stored row-major like K and never transposed in
// memory.
#include <math.h>

#include "common.h"

namespace dfs {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int KN = 64;   // key rows per LDS tile

__device__ __forceinline__ int block_real_rows(int blk, int B, int M_v, int64_t N_v, int n_text) {
  int64_t real = blk < M_v ? N_v - int64_t(blk) * B : int64_t(n_text) - int64_t(blk - M_v) * B;
  return real >= B ? B : (real <= 0 ? 0 : int(real));
}

template <int D, int BM>
__global__ void __launch_bounds__(BM * 2) __attribute__((amdgpu_waves_per_eu(2, 2)))
attn_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                 const int32_t* __restrict__ kv_idx, const int32_t* __restrict__ kv_cnt, int K_max, uint16_t* __restrict__ o,
                 float* __restrict__ lse, int64_t N_pad, int64_t N_v, int n_text, int M_v, int M, int total_wg,
                 int wg_per_xcd, float scale) {
  constexpr int NT = BM * 2;                       // threads: one wave per 32 query rows
  constexpr int KS = D + 8;                        // K tile row stride (elements): 16 B skew per row
  constexpr int VS = D + 32;                       // V tile row stride: 64 B skew per row
  constexpr int CH = D / 8;                        // 16-byte chunks per row
  constexpr int LD = KN * CH / NT;                 // chunks each thread stages per tile
  constexpr int STEPS = BM / KN;                   // tiles per key block
  __shared__ __attribute__((aligned(16))) uint16_t sK[KN * KS];
  __shared__ __attribute__((aligned(16))) uint16_t sV[KN * VS];

  // Work-group to (head, query block): consecutive ids on one XCD (ids are dealt round-robin to the
  // 8 XCDs) walk the query blocks of one head, so neighbouring blocks share key blocks in that
  // XCD's L2.  Query blocks are taken last-first: the dense text blocks at the end start first.
  const int logical = (blockIdx.x % 8) * wg_per_xcd + blockIdx.x / 8;
  if (logical >= total_wg) return;
  const int head = logical / M;
  const int u = M - 1 - logical % M;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int cnt_in = kv_cnt[int64_t(head) * M + u];
  const bool dense = cnt_in >= M;
  const int cnt = dense ? M : (cnt_in < 0 ? 0 : (cnt_in > K_max ? K_max : cnt_in));
  const int32_t* idx = kv_idx + (int64_t(head) * M + u) * K_max;
  const int64_t head_off = int64_t(head) * N_pad * D;
  const uint16_t* kh = k + head_off;
  const uint16_t* vh = v + head_off;
  const int64_t q_row = int64_t(u) * BM + wave * 32 + n;

  // Q rows as the B operand of S^T = K Q^T: lane (n, h) holds Q[row n][16 kk + 8 h .. + 7]
  bf16x8 qf[D / 16];
  {
    const u32x4* qp = reinterpret_cast<const u32x4*>(q + head_off + q_row * D);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, qp[2 * kk + h]);
  }

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = scale * 1.4426950408889634f;     // softmax in base 2

  const int n_tiles = cnt * STEPS;
  u32x4 pk[LD], pv[LD];
  auto fetch = [&](int tile) {
    int blk = dense ? tile / STEPS : idx[tile / STEPS];
    blk = unsigned(blk) < unsigned(M) ? blk : 0;      // a corrupt list must not read out of bounds
    const int64_t row0 = int64_t(blk) * BM + (tile % STEPS) * KN;
    const u32x4* ks = reinterpret_cast<const u32x4*>(kh + row0 * D);
    const u32x4* vs = reinterpret_cast<const u32x4*>(vh + row0 * D);
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      pk[i] = ks[tid + i * NT];
      pv[i] = vs[tid + i * NT];
    }
    return blk;
  };
  int blk_next = 0;
  if (n_tiles > 0) blk_next = fetch(0);

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int blk = blk_next;
    __syncthreads();                                 // every wave is done with the previous tile
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      const int c = tid + i * NT;
      const int row = c / CH, col = c % CH;
      *reinterpret_cast<u32x4*>(&sK[row * KS + col * 8]) = pk[i];
      *reinterpret_cast<u32x4*>(&sV[row * VS + col * 8]) = pv[i];
    }
    __syncthreads();
    if (tile + 1 < n_tiles) blk_next = fetch(tile + 1);

    // S^T tile pair: st[t][i] = logit(key row 32 t + 8 (i/4) + 4 h + i%4, query row n)
    f32x16 st[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int i = 0; i < 16; ++i) st[t][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&sK[(32 * t + n) * KS + 16 * kk + 8 * h]));
        st[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], st[t], 0, 0, 0);
      }
    }
    const int real = block_real_rows(blk, BM, M_v, N_v, n_text);
    if (real < BM) {                                  // ragged last block: pad keys never count
      const int base = (tile % STEPS) * KN;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (base + 32 * t + 8 * (i / 4) + 4 * h + (i % 4) >= real) st[t][i] = -INFINITY;
    }

    // online softmax for query row n (this lane and lane^32 hold the two halves of its keys)
    float mx = st[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, st[t][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;   // a row that has seen only pad keys
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * c2);
    const float mc = m_use * c2;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(st[t][i], c2, -mc));
        psum += p;
        pf[2 * t + i / 8][i % 8] = (__bf16)p;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;

    // O^T += V^T P^T.  Product step s covers key rows 16 s + {4h..4h+3} and 16 s + 8 + {4h..4h+3},
    // which is what registers 8 (s%2) .. 8 (s%2) + 7 of st[s/2] hold; the transposing LDS read hands
    // each lane four consecutive key rows of one value column.
    const int vrow = 4 * h + ((lane & 15) >> 2);
    const int vcol = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint16_t* p0 = &sV[(16 * s + vrow) * VS + dt * 32 + vcol];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p0 + 8 * VS));
        const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[s], oacc[dt], 0, 0, 0);
      }
    }
  }

  // epilogue: normalise, round to bf16, store.  Lane (n, h) holds O[row n][32 dt + 8 j + 4 h + 0..3].
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  uint16_t* orow = o + head_off + q_row * D;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[dt][4 * j + e] * inv);
      *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * j + 4 * h) = __builtin_bit_cast(u32x2, w);
    }
  if (lse && h == 0)
    lse[int64_t(head) * N_pad + q_row] = l_tot > 0.f ? (m_run * c2 + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
}

// ---------------------------------------------------------------------------------------------
// fp32 kernel: correctness path for fp32 tensors (small problems).  One thread per query row, key
// and value rows broadcast from LDS in tiles of 16, plain fp32 FMA, softmax rescaled once per tile.
template <int D>
__global__ void __launch_bounds__(128) attn_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                       const float* __restrict__ v, const int32_t* __restrict__ kv_idx,
                                                       const int32_t* __restrict__ kv_cnt, int K_max, float* __restrict__ o,
                                                       float* __restrict__ lse, int64_t N_pad, int64_t N_v, int n_text, int M_v,
                                                       int M, int B, float scale) {
  constexpr int TR = 16;
  __shared__ __attribute__((aligned(16))) float sK[TR * D];
  __shared__ __attribute__((aligned(16))) float sV[TR * D];
  const int head = blockIdx.y, u = blockIdx.x, tid = threadIdx.x;
  const int cnt_in = kv_cnt[int64_t(head) * M + u];
  const bool dense = cnt_in >= M;
  const int cnt = dense ? M : (cnt_in < 0 ? 0 : (cnt_in > K_max ? K_max : cnt_in));
  const int32_t* idx = kv_idx + (int64_t(head) * M + u) * K_max;
  const int64_t head_off = int64_t(head) * N_pad * D;
  const int64_t q_row = int64_t(u) * B + tid;
  float qr[D], acc[D];
  const f32x4* qp = reinterpret_cast<const f32x4*>(q + head_off + q_row * D);
#pragma unroll
  for (int c = 0; c < D / 4; ++c) {
    const f32x4 t = qp[c];
    qr[4 * c] = t[0] * scale; qr[4 * c + 1] = t[1] * scale; qr[4 * c + 2] = t[2] * scale; qr[4 * c + 3] = t[3] * scale;
  }
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  for (int it = 0; it < cnt; ++it) {
    int blk = dense ? it : idx[it];
    blk = unsigned(blk) < unsigned(M) ? blk : 0;
    const int real = block_real_rows(blk, B, M_v, N_v, n_text);
    for (int r0 = 0; r0 < real; r0 += TR) {
      const int rows = real - r0 < TR ? real - r0 : TR;
      __syncthreads();
      const f32x4* ks = reinterpret_cast<const f32x4*>(k + head_off + (int64_t(blk) * B + r0) * D);
      const f32x4* vs = reinterpret_cast<const f32x4*>(v + head_off + (int64_t(blk) * B + r0) * D);
      for (int c = tid; c < rows * (D / 4); c += B) {
        reinterpret_cast<f32x4*>(sK)[c] = ks[c];
        reinterpret_cast<f32x4*>(sV)[c] = vs[c];
      }
      __syncthreads();
      float s[TR];
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < TR; ++j) {
        float d0 = 0.f;
        if (j < rows) {
#pragma unroll
          for (int c = 0; c < D; ++c) d0 = fmaf(qr[c], sK[j * D + c], d0);
        } else {
          d0 = -INFINITY;
        }
        s[j] = d0;
        mx = fmaxf(mx, d0);
      }
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __expf(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] *= alpha;
#pragma unroll
      for (int j = 0; j < TR; ++j) {
        if (j < rows) {
          const float p = __expf(s[j] - m_new);
          l_run += p;
#pragma unroll
          for (int c = 0; c < D; ++c) acc[c] = fmaf(p, sV[j * D + c], acc[c]);
        }
      }
      m_run = m_new;
    }
  }
  const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
  f32x4* op = reinterpret_cast<f32x4*>(o + head_off + q_row * D);
#pragma unroll
  for (int c = 0; c < D / 4; ++c) op[c] = f32x4{acc[4 * c] * inv, acc[4 * c + 1] * inv, acc[4 * c + 2] * inv, acc[4 * c + 3] * inv};
  if (lse) lse[int64_t(head) * N_pad + q_row] = l_run > 0.f ? m_run + __logf(l_run) : -INFINITY;
}

int run_sparse_attn(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q, const void* k, const void* v,
                    const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale, void* o, float* lse,
                    hipStream_t st) {
  if (K_max < 1) return fail(DFS_ESHAPE, "dfs_sparse_attn_fwd: K_max=%d must be positive", K_max);
  if (dtype == DFS_BF16) {
    const int64_t total = int64_t(g->heads) * s.M;
    if (total > (int64_t(1) << 30)) return fail(DFS_ESHAPE, "dfs_sparse_attn_fwd: heads*M too large");
    const int per_xcd = int((total + 7) / 8);
    dim3 grid(unsigned(per_xcd * 8));
#define ATTN(DD, BB)                                                                                                        \
  attn_bf16_kernel<DD, BB><<<grid, BB * 2, 0, st>>>(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),        \
                                                    static_cast<const uint16_t*>(v), kv_idx, kv_cnt, K_max,                  \
                                                    static_cast<uint16_t*>(o), lse, s.N_pad, s.N_v, g->n_text, s.M_v, s.M,   \
                                                    int(total), per_xcd, scale)
    if (g->d == 64) { if (g->B == 64) ATTN(64, 64); else ATTN(64, 128); }
    else            { if (g->B == 64) ATTN(128, 64); else ATTN(128, 128); }
#undef ATTN
  } else {
    if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
    dim3 grid(unsigned(s.M), unsigned(g->heads));
    if (g->d == 64)
      attn_f32_kernel<64><<<grid, g->B, 0, st>>>(static_cast<const float*>(q), static_cast<const float*>(k),
                                                 static_cast<const float*>(v), kv_idx, kv_cnt, K_max, static_cast<float*>(o), lse,
                                                 s.N_pad, s.N_v, g->n_text, s.M_v, s.M, g->B, scale);
    else
      attn_f32_kernel<128><<<grid, g->B, 0, st>>>(static_cast<const float*>(q), static_cast<const float*>(k),
                                                  static_cast<const float*>(v), kv_idx, kv_cnt, K_max, static_cast<float*>(o), lse,
                                                  s.N_pad, s.N_v, g->n_text, s.M_v, s.M, g->B, scale);
  }
  return launch_status("dfs_sparse_attn_fwd");
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_sparse_attn_fwd(const dfs_geom* g, int dtype, const void* q_perm, const void* k_perm, const void* v_perm,
                                   const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale, void* o_perm,
                                   float* lse, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_F32 && dtype != DFS_BF16) return fail(DFS_EDTYPE, "dtype %d is not DFS_F32 or DFS_BF16", dtype);
  if (!q_perm || !k_perm || !v_perm || !kv_idx || !kv_cnt || !o_perm) return fail(DFS_EINVAL, "dfs_sparse_attn_fwd: NULL argument");
  if (!(scale > 0.f)) return fail(DFS_EINVAL, "dfs_sparse_attn_fwd: scale must be positive");
  return run_sparse_attn(g, s, dtype, q_perm, k_perm, v_perm, kv_idx, kv_cnt, K_max, scale, o_perm, lse, as_stream(stream));
}
