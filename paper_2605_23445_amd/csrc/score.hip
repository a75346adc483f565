// Hierarchical block scoring (paper Sec. 5.2; Algorithm 1 step 2; Eq. 2 and Eq. 8).
//
//   pool_kernel   : Q_hat, K_hat = mean over the real rows of each sub-block, an HBM stream.  The fp32
//                   means (Q_hat already times 1/sqrt(d)) are scaled, four consecutive sub-blocks at a time,
//                   by the power of two that brings their largest magnitude to 2^11..2^12, and stored as two
//                   fp16 terms x = hi + lo, which together carry 22 bits of the value.
//   score_lse_kernel / score_fold_kernel : S_hat[u,v] = sum over the r x r sub-block pairs of
//                   softmax(Q_hat K_hat^T / sqrt(d)).  The sub-block attention matrix A_hat is never stored.
//                   One pass over the contraction: per (query sub-block, key block) the base-2 log of the
//                   summed exponentials of the block's key sub-blocks and per query sub-block the row
//                   log-sum-exp; a second, memory-bound kernel turns these into probabilities and folds the r
//                   query sub-blocks of a query block.  The logits run on the fp16 matrix cores as three
//                   partial products hi.hi + hi.lo + lo.hi with fp32 accumulation: every fp16 product is exact
//                   in fp32 and the dropped lo.lo term is below 2^-22 of the result, so the logits are as
//                   accurate as an fp32 contraction at several times its speed (the mask decision that
//                   follows stays an fp32 one); the scaling is undone, exactly, on the fp32 result.
#include <type_traits>

#include "common.h"

namespace dfs {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------ pooling

// x (already scaled so that its group's largest magnitude is in [2^11, 2^12)) -> (hi, lo) with hi = fp16(x),
// lo = fp16(x - hi).  The subtraction is exact and |x - hi| <= 2^-11 |x|, so x = hi + lo to within 2^-22 |x| as long
// as lo is a normal fp16 number, which it is for |x| >= 2^-3: an element more than 2^14 times smaller than the
// largest of its group is kept to 2^-25 absolute instead, i.e. to 2^-36 of that largest one.
__device__ __forceinline__ void split2(float x, uint16_t& hi, uint16_t& lo) {
  const _Float16 h = (_Float16)x;
  const _Float16 l = (_Float16)(x - (float)h);
  hi = __builtin_bit_cast(uint16_t, h);
  lo = __builtin_bit_cast(uint16_t, l);
}
// Rows are scaled in groups of four consecutive sub-blocks (the four waves of a pooling work-group) by a power of
// two that brings the group's largest magnitude into [2^11, 2^12); `down` is the inverse.  Powers of two: exact.
constexpr int SHIFT_MAX = 126;                 // keeps both factors finite and normal for groups of vanishing magnitude
                                               // (the largest finite fp32 needs a shift of -116)
__device__ __forceinline__ void group_scale(float gmax, float& up, float& down) {
  up = 1.0f; down = 1.0f;
  if (gmax > 0.f && gmax < INFINITY) {
    int ex;
    (void)frexpf(gmax, &ex);                   // gmax = m 2^ex, m in [0.5, 1)
    int sh = 12 - ex;
    sh = sh > SHIFT_MAX ? SHIFT_MAX : (sh < -SHIFT_MAX ? -SHIFT_MAX : sh);
    up = ldexpf(1.0f, sh);
    down = ldexpf(1.0f, -sh);
  }
}

// One wave per sub-block.  Lanes of a row sit side by side (16 bytes each); several rows are in
// flight per load; partial sums of the row groups are folded with cross-lane exchanges.
// Output row layout: [2][D] fp16 (hi, lo planes) of the row times its group's scale; the inverse scale of
// group s / 4 goes to q_down / k_down.
template <bool BF16, int D>
__global__ void __launch_bounds__(256) pool_kernel(const void* __restrict__ q_perm, const void* __restrict__ k_perm,
                                                   uint16_t* __restrict__ q_hat, uint16_t* __restrict__ k_hat,
                                                   float* __restrict__ q_down, float* __restrict__ k_down,
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
  const bool pooled = s < M_s;                               // this wave has a sub-block to pool
  const bool busy = pooled || (k_copy && int64_t(s) * Bs < N_pad);
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
  const int rows = !busy ? 0 : k_copy ? Bs : cnt;   // a copy covers the pad rows of the sub-block as well
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
#pragma unroll
  for (int off = TPR; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
  }
  // every lane now holds the column sums of its 16 bytes of the row; the row's largest magnitude, then the group's
  const float inv = pooled && cnt > 0 ? (blockIdx.z == 0 ? q_scale : 1.0f) / float(cnt) : 0.f;
  float mx = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    acc[e] *= inv;
    mx = fmaxf(mx, fabsf(acc[e]));
  }
#pragma unroll
  for (int off = 1; off < TPR; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  __shared__ float s_max[4];
  if (lane == 0) s_max[threadIdx.x >> 6] = mx;
  __syncthreads();                             // reached by all four waves: none has left the kernel
  if (!pooled) return;                         // copied only, or beyond the last sub-block
  float up, down;
  group_scale(fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3])), up, down);
  if (threadIdx.x == 0) (blockIdx.z == 0 ? q_down : k_down)[int64_t(head) * ((M_s + 3) / 4) + blockIdx.x] = down;
  if (rg == 0) {
    uint16_t* o = dst + (int64_t(head) * M_s + s) * (2 * D) + c * EPL;
    uint16_t hi[EPL], lo[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) split2(acc[e] * up, hi[e], lo[e]);
#pragma unroll
    for (int e = 0; e < EPL; e += 2) {
      *reinterpret_cast<uint32_t*>(o + e) = uint32_t(hi[e]) | (uint32_t(hi[e + 1]) << 16);
      *reinterpret_cast<uint32_t*>(o + D + e) = uint32_t(lo[e]) | (uint32_t(lo[e + 1]) << 16);
    }
  }
}

// ------------------------------------------------------------------------------------ scoring

// T is stored with its rows padded to whole query groups (128 sub-blocks) and its row count to whole key tiles,
// so that the contraction kernel stores without a bounds check: [heads][t_rows][t_cols] fp32.
__host__ __device__ inline int t_cols(int M_s) { return (M_s + 127) / 128 * 128; }
__host__ __device__ inline int t_rows(int M_s, int R) { return (M_s + 31) / 32 * (32 / R); }

constexpr float LSE_START = -1.0e30f;          // finite stand-in for "nothing seen yet" (keeps differences finite)

__device__ __forceinline__ float vmax3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// The value of the other lane half (lane ^ 32) beside this lane's own, through the vector unit (a shuffle through
// LDS would make the wave wait for every LDS read in flight).  Returns {lower half's value, upper half's value}.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  lo = __uint_as_float(sw[0]);
  hi = __uint_as_float(sw[1]);
}

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
score_lse_kernel(const uint16_t* __restrict__ q_hat, const uint16_t* __restrict__ k_hat, const float* __restrict__ q_down,
                 const float* __restrict__ k_down, float* __restrict__ tt, float* __restrict__ lse, int M_s, int n_live, int tiles_per_split, int ksplit,
                 int wgs_per_head, int total_wgs, int wgs_per_xcd) {
  constexpr int RS = 2 * D;                   // elements of a centroid row (hi, lo planes)
  constexpr int RSP = RS + 8;                 // LDS row stride: 16 bytes of skew keep the row-per-lane reads conflict-free
  constexpr int KS = D / 16;                  // product steps of 16 features
  constexpr int CPT = 32 * RS / 8 / 256;      // 16-byte chunks of a key tile per thread (6 at d=128)
  constexpr int G = R < 4 ? R : 4;            // key sub-blocks of one key block that sit in consecutive registers
  __shared__ __attribute__((aligned(16))) uint16_t s_k[2][32 * RSP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  // Work-group ids are dealt round-robin to the 8 XCDs, each with an L2 of its own.  Every XCD takes a contiguous
  // eighth of the (head, query group, key range) list, so that the work-groups resident on an XCD belong to one or
  // two heads and that head's key centroids (re-read by every one of them) stay in its L2.
  const int logical = (blockIdx.x % 8) * wgs_per_xcd + blockIdx.x / 8;
  if (logical >= total_wgs) return;           // the whole work-group: no barrier has been reached yet
  const int head = logical / wgs_per_head, in_head = logical % wgs_per_head;
  const int split = in_head % ksplit;
  const int i0 = (in_head / ksplit) * 128 + wave * 32;      // first query sub-block of this wave
  const uint16_t* qh = q_hat + int64_t(head) * M_s * RS;
  const uint16_t* kh = k_hat + int64_t(head) * M_s * RS;

  // Query centroids as the B operand: lane (n, half) holds row i0 + n, features 16 kk + 8 half .. + 7, two planes.
  const int G4 = (M_s + 3) / 4;               // scale groups (four consecutive sub-blocks) per head
  f16x8 bq[2][KS];
  float q_dn = 1.0f;                          // inverse scale of this lane's query row
  {
    const int row = i0 + n;
    if (row < M_s) q_dn = q_down[int64_t(head) * G4 + row / 4];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (row < M_s) v = *reinterpret_cast<const u32x4*>(qh + int64_t(row) * RS + p * D + 16 * kk + 8 * half);
        bq[p][kk] = __builtin_bit_cast(f16x8, v);
      }
  }
  const int n_tiles = (n_live + 31) / 32;     // key sub-blocks at or beyond n_live are empty
  const int t_begin = split * tiles_per_split;
  const int t_end = t_begin + tiles_per_split < n_tiles ? t_begin + tiles_per_split : n_tiles;

  // key tile t (32 centroid rows, contiguous in memory) -> registers -> LDS
  u32x4 kreg[CPT];
  auto fetch = [&](int t) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      // rows at or beyond M_s re-read the last row instead (no branch): they are at or beyond n_live and masked later
      const int c = tid + i * 256;
      const int row = t * 32 + c / (RS / 8);
      const int from = row < M_s ? row : M_s - 1;
      kreg[i] = *reinterpret_cast<const u32x4*>(kh + int64_t(from) * RS + (c % (RS / 8)) * 8);
    }
  };
  auto commit = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<u32x4*>(&s_k[buf][(c / (RS / 8)) * RSP + (c % (RS / 8)) * 8]) = kreg[i];
    }
  };
  float m_row = LSE_START, z_row = 0.f;       // this lane's share of the row log-sum-exp of query sub-block i0 + n
  const int q_row = i0 + n;
  const int TC = t_cols(M_s);
  float* tt_h = tt + int64_t(head) * t_rows(M_s, R) * TC;
  const int t_lane = (R == 8 ? 0 : half) * (R == 1 ? 4 : R == 2 ? 2 : 1) * TC + q_row;   // this lane's share of a T index
  // inverse scales for the four row groups of tile t that this lane's registers cover, times the query row's
  auto load_dn = [&](int t, float (&dn)[4]) {
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {            // scale group of key rows 32 t + 8 gq + 4 half .. + 3
      const int grp = 8 * t + 2 * gq + half;
      dn[gq] = k_down[int64_t(head) * G4 + (grp < G4 ? grp : G4 - 1)] * q_dn;     // beyond the last group: masked rows
    }
  };

  // One pipeline stage, written out in issue order: the matrix instructions of tile t and, in their shadow, the
  // epilogue of the tile before, cut into 24 slices.  (Two waves of a SIMD that each run their matrix phase and
  // then their vector phase fall into step, and the two kinds of work then add up instead of overlapping.)
  //   matrix part: transposed logits of the 32 x 32 tile, a[i] = <k_hat[row 8 (i/4) + 4 half + i%4 of the tile],
  //     q_hat[i0 + n]>, as hi.hi + hi.lo + lo.hi products (lo.lo is below 2^-22 of the result) with fp32
  //     accumulation, dealt to two accumulators c0, c1 in turn so that no matrix instruction waits for the one
  //     before it; the operands of two product steps are requested from LDS one pair ahead; tile t + 1 goes from
  //     its staging registers to LDS early in the stage, and only then the loads of tile t + 2 are issued, so
  //     they have a whole stage to land.
  //   epilogue of tile tp from its accumulators p0, p1: logits = (p0 + p1) x inverse scales (registers 4 g .. 4 g + 3
  //     of a lane are four consecutive key rows, one scale group); one reference for the whole tile, the running
  //     row maximum including this tile (finite from the start, so no difference is ever inf - inf; masked logits
  //     give 2^-inf = 0; R == 8: a key block is split over the two lane halves, which therefore share the
  //     reference); then per key block the log of its summed exponentials.
  constexpr int NS = 3 * KS;                  // matrix instructions of a tile
  auto stage = [&](auto do_mm, auto do_ep, int t, int buf, f32x16& c0, f32x16& c1, float (&dn_next)[4], const f32x16& p0,
                   const f32x16& p1, const float (&dn_prev)[4], int tp) {
    constexpr bool MM = decltype(do_mm)::value, EP = decltype(do_ep)::value;
    const uint16_t* krow = &s_k[buf][n * RSP + 8 * half];
    f16x8 fr[2][4];
    auto load_pair = [&](int p) {
      fr[p & 1][0] = __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(krow + 32 * p));
      fr[p & 1][1] = __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(krow + D + 32 * p));
      fr[p & 1][2] = __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(krow + 32 * p + 16));
      fr[p & 1][3] = __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(krow + D + 32 * p + 16));
    };
    float dp[4], c[16];
    float mt = 0.f, m_new = 0.f, zt = 0.f;
    if (EP) {
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) dp[gq] = dn_prev[gq];      // dn_next may be the same array
    }
    if (MM) {
      load_pair(0);
#pragma unroll
      for (int i = 0; i < 16; ++i) { c0[i] = 0.f; c1[i] = 0.f; }
    }
    auto slice = [&](int sl) {
      if (sl < 8) {
#pragma unroll
        for (int i = 2 * sl; i < 2 * sl + 2; ++i) c[i] = (p0[i] + p1[i]) * dp[i / 4];
      } else if (sl == 8) {
        if (__builtin_expect(tp * 32 + 32 > n_live, 0)) {   // ragged end: key sub-blocks without rows count for nothing
          asm volatile("");                   // keeps this a branch: as selects it would run on every tile
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (tp * 32 + 8 * (i / 4) + 4 * half + (i % 4) >= n_live) c[i] = -INFINITY;
        }
        mt = vmax3(c[0], c[1], c[2]);
      } else if (sl < 12) {
        const int i = 3 + 4 * (sl - 9);
        mt = vmax3(mt, c[i], c[i + 1]);
        mt = vmax3(mt, c[i + 2], c[i + 3]);
      } else if (sl == 12) {
        mt = fmaxf(mt, c[15]);
        if (R == 8) {
          float lo, hi;
          both_halves(mt, lo, hi);
          mt = fmaxf(lo, hi);
        }
        m_new = fmaxf(m_row, mt);
        z_row *= __builtin_amdgcn_exp2f(m_row - m_new);
        m_row = m_new;
      } else {
        if (sl < 21) {
#pragma unroll
          for (int i = 2 * (sl - 13); i < 2 * (sl - 13) + 2; ++i) {
            const float e = __builtin_amdgcn_exp2f(c[i] - m_new);
            if (G == 1) zt += e; else c[i] = e;
          }
        }
        if (sl >= 20) {
          // fold the key sub-blocks of each key block: groups of G consecutive registers
          constexpr int NG = 16 / G;
#pragma unroll
          for (int gi = (sl - 20) * NG / 4; gi < (sl - 19) * NG / 4; ++gi) {
            float tv;
            if (G == 1) {
              tv = c[gi];
            } else {
              float sg = 0.f;
#pragma unroll
              for (int e = 0; e < G; ++e) sg += c[gi * G + e];
              zt += sg;                        // this lane's own share of the row sum
              if (R == 8) {
                float lo, hi;
                both_halves(sg, lo, hi);
                sg = lo + hi;
              }
              // a block whose sum vanishes against the row maximum (below 2^-126 of it) scores nothing: log2(0) = -inf
              tv = m_new + __builtin_amdgcn_logf(sg);
            }
            // key sub-block of the group's first register: 8 (first / 4) + 4 half + first % 4
            // key block = (32 tp + 8 (first / 4) + first % 4) / R + the lane half's share, which is in t_lane; the
            // uniform part goes into a scalar base.  No bounds check: T is padded, and at R = 8 both lane halves
            // store the same value to the same place.
            const int first = gi * G;
            const int v_uniform = (tp * 32 + 8 * (first / 4) + (first % 4)) / R;
            (tt_h + int64_t(v_uniform) * TC)[t_lane] = tv;
          }
          if (sl == 23) z_row += zt;
        }
      }
    };
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < NS; ++m) {
      if (MM) {
        const int p = m / 6, j = m % 6, kk = 2 * p;
        if (j == 0 && p + 1 < KS / 2) load_pair(p + 1);
        const f16x8(&f)[4] = fr[p & 1];
        if (j == 0) c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[0], bq[0][kk], c0, 0, 0, 0);          // hi.hi
        if (j == 1) c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[0], bq[1][kk], c1, 0, 0, 0);          // hi.lo
        if (j == 2) c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[1], bq[0][kk], c0, 0, 0, 0);          // lo.hi
        if (j == 3) c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[2], bq[0][kk + 1], c1, 0, 0, 0);
        if (j == 4) c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[2], bq[1][kk + 1], c0, 0, 0, 0);
        if (j == 5) c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[3], bq[0][kk + 1], c1, 0, 0, 0);
        if (m == 2 && t + 1 < t_end) commit(buf ^ 1);      // the other buffer was last read before the previous barrier
        if (m == 4 && t + 2 < t_end) fetch(t + 2);
        if (m == NS / 2 && t + 1 < t_end) load_dn(t + 1, dn_next);   // the epilogue is done with dn_prev by now
      }
      if (EP) {
#pragma unroll
        for (int sl = m * 24 / NS; sl < (m + 1) * 24 / NS; ++sl) slice(sl);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MM) __syncthreads();                  // tile t has been read by every wave; tile t + 1 is in LDS
  };

  if (t_begin < t_end) {
    using yes = std::true_type;
    using no = std::false_type;
    // tiles alternate between two sets of accumulators and inverse scales (the second set is handed, unused, to the
    // first stage, which has no epilogue)
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 xa0 = zero16, xa1 = zero16, ya0 = zero16, ya1 = zero16;
    float dx[4] = {1.f, 1.f, 1.f, 1.f}, dy[4] = {1.f, 1.f, 1.f, 1.f};
    load_dn(t_begin, dx);
    fetch(t_begin);
    commit(0);
    if (t_begin + 1 < t_end) fetch(t_begin + 1);
    __syncthreads();
    int t = t_begin;
    stage(yes{}, no{}, t, 0, xa0, xa1, dy, ya0, ya1, dy, t);
    ++t;
    for (; t + 1 < t_end; t += 2) {
      stage(yes{}, yes{}, t, 1, ya0, ya1, dx, xa0, xa1, dx, t - 1);
      stage(yes{}, yes{}, t + 1, 0, xa0, xa1, dy, ya0, ya1, dy, t);
    }
    if (t < t_end) {
      stage(yes{}, yes{}, t, 1, ya0, ya1, dx, xa0, xa1, dx, t - 1);
      stage(no{}, yes{}, t, 0, xa0, xa1, dx, ya0, ya1, dy, t);
    } else {
      stage(no{}, yes{}, t, 0, ya0, ya1, dy, xa0, xa1, dx, t - 1);
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
  const int TC = t_cols(M_s);
  const float* tt_h = tt + int64_t(head) * t_rows(M_s, R) * TC;
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
      const float* row = tt_h + int64_t(v) * TC + int64_t(u0 + tx) * R;
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

// Workspace: Q_hat, K_hat (two fp16 planes each, followed by the inverse scales of their row groups),
// T [heads][t_rows][t_cols] fp32 (padded, see t_cols), row log-sum-exp [heads][KSPLIT_MAX][M_s] fp32.
constexpr int KSPLIT_MAX = 4;
static size_t ws_planes_bytes(const dfs_geom* g, const dfs_sizes& s) { return align256(size_t(g->heads) * s.M_s * 2 * g->d * sizeof(uint16_t)); }
static size_t ws_hat_bytes(const dfs_geom* g, const dfs_sizes& s) {
  return ws_planes_bytes(g, s) + align256(size_t(g->heads) * ((s.M_s + 3) / 4) * sizeof(float));
}
static size_t ws_tt_bytes(const dfs_geom* g, const dfs_sizes& s) {
  return align256(size_t(g->heads) * t_rows(s.M_s, s.r) * t_cols(s.M_s) * sizeof(float));
}
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
static void launch_score(const dfs_geom* g, const dfs_sizes& s, const uint16_t* q_hat, const uint16_t* k_hat, const float* q_down,
                         const float* k_down, float* tt, float* lse, float* score, int n_live, hipStream_t st) {
  const int groups = (s.M_s + 127) / 128, n_tiles = (n_live + 31) / 32;
  const int ksplit = choose_ksplit(int64_t(groups) * g->heads, n_tiles);
  const int per = (n_tiles + ksplit - 1) / ksplit;
  const int wgs_per_head = groups * ksplit;
  const int64_t total = int64_t(wgs_per_head) * g->heads;
  const int per_xcd = int((total + 7) / 8);
  score_lse_kernel<D, R><<<dim3(unsigned(per_xcd * 8)), 256, 0, st>>>(q_hat, k_hat, q_down, k_down, tt, lse, s.M_s, n_live, per, ksplit,
                                                                      wgs_per_head, int(total), per_xcd);
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
  float* q_down = reinterpret_cast<float*>(base + ws_planes_bytes(g, s));
  float* k_down = reinterpret_cast<float*>(base + ws_hat_bytes(g, s) + ws_planes_bytes(g, s));
  float* tt = reinterpret_cast<float*>(base + 2 * ws_hat_bytes(g, s));
  float* lse = reinterpret_cast<float*>(base + 2 * ws_hat_bytes(g, s) + ws_tt_bytes(g, s));
  const int64_t pool_subs = k_out ? s.N_pad / g->Bs : s.M_s;   // with k_out the text blocks are copied as well
  dim3 pg(unsigned((pool_subs + 3) / 4), unsigned(g->heads), 2);
  const bool bf = dtype == DFS_BF16;
  // 1/sqrt(d) of Eq. 2 and the change to base 2 go into Q_hat, so that the logits come out of the contraction in base 2
  const float scale = 1.4426950408889634f / sqrtf(float(g->d));
#define POOL(BF, DD) pool_kernel<BF, DD><<<pg, 256, 0, st>>>(q_perm, k_perm, q_hat, k_hat, q_down, k_down, q_index, k_out, s.N, s.N_pad, s.N_v, g->Bs, s.M_s, scale)
  if (g->d == 64) { if (bf) POOL(true, 64); else POOL(false, 64); }
  else            { if (bf) POOL(true, 128); else POOL(false, 128); }
#undef POOL
  const int n_live = int((s.N_v + g->Bs - 1) / g->Bs);
#define SCORE(DD, RR) launch_score<DD, RR>(g, s, q_hat, k_hat, q_down, k_down, tt, lse, score, n_live, st)
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
