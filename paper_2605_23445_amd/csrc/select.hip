// Block-mask selection (paper Eq. 9) and the cumulative-mass keep count.
//
// One wave owns one (head, query block) row of scores.  Scores are mapped to 32-bit keys whose
// unsigned order is the float order; the k-th largest key is found a byte at a time from the top (four
// histogram passes over the row in LDS), ties at the threshold are resolved towards the lower
// column index, and the kept columns are written in ascending order with ballot prefix sums.
// Everything is integer work on the bit patterns, so the result is exactly the total order
// "higher score first, equal scores by lower index".
#include <math.h>

#include <mutex>

#include "common.h"

namespace dfs {

// Scratch of dfs_select_mask_static: the per-row and per-head keep counts of the mass modes live here instead
// of in a caller-supplied workspace.  One copy per GPU, held until the process ends.  Host code never uses the
// symbol's name as an address: the device address is resolved once per device (static_scratch below).
constexpr size_t STATIC_SCRATCH_BYTES = size_t(1) << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MASS_FRAC_BITS = 24;

__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t b = __float_as_uint(s);
  if (b == 0x80000000u) b = 0u;                     // -0 ranks with +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t lo = __shfl_xor(uint32_t(v), off, 64), hi = __shfl_xor(uint32_t(v >> 32), off, 64);
    v += (static_cast<unsigned long long>(hi) << 32) | lo;
  }
  return v;
}

__device__ __forceinline__ unsigned long long mass_fixed(float s) {
  const double c = fmin(fmax(double(s), 0.0), 4096.0);   // NaN clamps to 0
  return static_cast<unsigned long long>(c * double(1 << MASS_FRAC_BITS));
}

// k_row[head, u] = fewest top-ranked columns whose fixed-point scores reach ceil(mass * row total).
__global__ void __launch_bounds__(64) mass_count_kernel(const float* __restrict__ score, int M_v, double mass,
                                                        int32_t* __restrict__ k_row) {
  extern __shared__ uint32_t keys[];
  const int lane = threadIdx.x;
  const float* row = score + (int64_t(blockIdx.y) * M_v + blockIdx.x) * M_v;
  unsigned long long tot = 0;
  for (int j = lane; j < M_v; j += 64) {
    const float s = row[j];
    keys[j] = order_key(s);
    tot += mass_fixed(s);
  }
  __syncthreads();
  tot = wave_sum_u64(tot);
  const unsigned long long target = static_cast<unsigned long long>(ceil(mass * double(tot)));
  int k = 1;
  if (target > 0) {
    // largest threshold T with sum over {key >= T} >= target
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = T | (1u << bit);
      unsigned long long part = 0;
      for (int j = lane; j < M_v; j += 64)
        if (keys[j] >= cand) part += mass_fixed(row[j]);
      if (wave_sum_u64(part) >= target) T = cand;
    }
    unsigned long long above = 0, at = 0;
    uint32_t n_above = 0;
    for (int j = lane; j < M_v; j += 64) {
      if (keys[j] > T) { above += mass_fixed(row[j]); ++n_above; }
      else if (keys[j] == T) at = mass_fixed(row[j]);
    }
    above = wave_sum_u64(above);
    n_above = wave_sum_u32(n_above);
    // every column at the threshold has the same fixed-point value; take the largest lane's copy
    unsigned long long at_all = at;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const uint32_t lo = __shfl_xor(uint32_t(at_all), off, 64), hi = __shfl_xor(uint32_t(at_all >> 32), off, 64);
      const unsigned long long o = (static_cast<unsigned long long>(hi) << 32) | lo;
      at_all = o > at_all ? o : at_all;
    }
    const unsigned long long need = target - above;          // > 0 by choice of T
    k = int(n_above + (need + at_all - 1) / at_all);
  }
  if (lane == 0) k_row[int64_t(blockIdx.y) * M_v + blockIdx.x] = k;
}

// k_head[h] = clamp(max(ceil(mean_u k_row[h,u]), k_floor), 1, k_cap)
__global__ void __launch_bounds__(256) head_count_kernel(const int32_t* __restrict__ k_row, int M_v, int k_floor, int k_cap,
                                                         int32_t* __restrict__ k_used, int32_t* __restrict__ k_head_out) {
  __shared__ unsigned long long part[4];
  unsigned long long s = 0;
  for (int u = threadIdx.x; u < M_v; u += 256) s += uint32_t(k_row[int64_t(blockIdx.x) * M_v + u]);
  s = wave_sum_u64(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned long long tot = part[0] + part[1] + part[2] + part[3];
    int k = int((tot + M_v - 1) / M_v);
    if (k < k_floor) k = k_floor;
    if (k > k_cap) k = k_cap;
    if (k < 1) k = 1;
    k_used[blockIdx.x] = k;
    if (k_head_out) k_head_out[blockIdx.x] = k;
  }
}

// Top-k of one row.  k is `k_fixed`, or k_per_head[head], or clamp(k_per_row[head, u], k_fixed, k_cap).
__global__ void __launch_bounds__(64) select_kernel(const float* __restrict__ score, int M_v, int M_x, int k_fixed,
                                                    const int32_t* __restrict__ k_per_head, const int32_t* __restrict__ k_per_row,
                                                    int k_cap, uint8_t* __restrict__ mask,
                                                    int32_t* __restrict__ kv_idx, int32_t* __restrict__ kv_cnt, int K_max,
                                                    int32_t* __restrict__ k_head_out) {
  extern __shared__ uint32_t keys[];
  const int lane = threadIdx.x;
  const int head = blockIdx.y, u = blockIdx.x;
  const int M = M_v + M_x;
  uint8_t* mrow = mask ? mask + (int64_t(head) * M + u) * M : nullptr;
  if (u >= M_v) {                                   // text query block: keeps every key block
    if (mrow)
      for (int j = lane; j < M; j += 64) mrow[j] = 1;
    if (lane == 0) kv_cnt[int64_t(head) * M + u] = M;
    return;
  }
  int k = k_per_head ? k_per_head[head] : k_fixed;
  if (k_per_row) {
    const int ku = k_per_row[int64_t(head) * M_v + u];
    k = ku < k_fixed ? k_fixed : (ku > k_cap ? k_cap : ku);
  }
  if (k_head_out && !k_per_head && !k_per_row && u == 0 && lane == 0) k_head_out[head] = k;
  const float* row = score + (int64_t(head) * M_v + u) * M_v;
  for (int j = lane; j < M_v; j += 64) keys[j] = order_key(row[j]);
  __syncthreads();
  // T = k-th largest key, found a byte at a time from the top: a 256-bin histogram of the next byte of the keys that
  // still match the bytes fixed so far, then the bin in which the count from the top reaches what is still wanted.
  // Four passes instead of one per bit; counts are integers, so the result is the same key.
  uint32_t* hist = keys + M_v;
  uint32_t T = 0, fixed = 0, want = uint32_t(k);      // want: rank of the key looked for among the keys matching T on `fixed`
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int b = lane; b < 256; b += 64) hist[b] = 0u;
    __syncthreads();
    for (int j = lane; j < M_v; j += 64) {
      const uint32_t key = keys[j];
      if ((key & fixed) == T) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    // lane l owns bins 255 - 4 l .. 252 - 4 l, so that lane order is descending key order
    uint32_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = hist[255 - 4 * lane - i];
    const uint32_t mine = c[0] + c[1] + c[2] + c[3];
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    const unsigned long long reached = __ballot(incl >= want);     // never empty: at least `want` keys match
    const int sel = __ffsll(reached) - 1;
    uint32_t left = want - (incl - mine), digit = 0u;              // meaningful in lane `sel` only
#pragma unroll
    for (int i = 3; i >= 0; --i) {                                 // the first bin (from the top) whose running count reaches `left`
      const uint32_t before = (i > 0 ? c[0] : 0u) + (i > 1 ? c[1] : 0u) + (i > 2 ? c[2] : 0u);
      if (before < left && left <= before + c[i]) digit = uint32_t(255 - 4 * lane - i) | ((left - before) << 8);
    }
    digit = __shfl(digit, sel, 64);
    T |= (digit & 255u) << shift;
    want = digit >> 8;
    fixed |= 255u << shift;
    __syncthreads();                                               // the histogram is cleared next
  }
  const uint32_t ties_wanted = want;                               // lowest-index columns equal to T; the k - want keys above T are all kept
  int32_t* idx = kv_idx + (int64_t(head) * M + u) * K_max;
  uint32_t ties_seen = 0, written = 0;
  const unsigned long long below_me = (1ull << lane) - 1ull;
  for (int j0 = 0; j0 < M_v; j0 += 64) {
    const int j = j0 + lane;
    const uint32_t key = j < M_v ? keys[j] : 0u;
    const bool is_tie = j < M_v && key == T;
    const unsigned long long tie_ballot = __ballot(is_tie);
    const uint32_t tie_rank = ties_seen + __popcll(tie_ballot & below_me);
    const bool keep = j < M_v && (key > T || (is_tie && tie_rank < ties_wanted));
    const unsigned long long keep_ballot = __ballot(keep);
    if (keep) idx[written + __popcll(keep_ballot & below_me)] = j;
    if (mrow && j < M_v) mrow[j] = keep ? 1 : 0;
    ties_seen += __popcll(tie_ballot);
    written += __popcll(keep_ballot);
  }
  for (int j = lane; j < M_x; j += 64) {             // text key blocks are always kept
    idx[k + j] = M_v + j;
    if (mrow) mrow[M_v + j] = 1;
  }
  if (lane == 0) kv_cnt[int64_t(head) * M + u] = k + M_x;
}

size_t ws_select_mask(const dfs_geom* g, const dfs_sizes& s) {
  return align256(size_t(g->heads) * s.M_v * sizeof(int32_t)) + align256(size_t(g->heads) * sizeof(int32_t));
}

int run_select_mask(const dfs_geom* g, const dfs_sizes& s, const float* score, int mode, double sparsity, double mass,
                    uint8_t* mask, int32_t* kv_idx, int32_t* kv_cnt, int32_t K_max, int32_t* k_head, void* ws,
                    hipStream_t st) {
  if (mode != DFS_SELECT_TOPK && mode != DFS_SELECT_MASS_HEAD && mode != DFS_SELECT_MASS_ROW)
    return fail(DFS_EINVAL, "dfs_select_mask: unknown mode %d", mode);
  if (!(sparsity >= 0.0 && sparsity <= 1.0)) return fail(DFS_EINVAL, "dfs_select_mask: sparsity %g is outside [0,1]", sparsity);
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  if (s.M_v > 16128) return fail(DFS_ESHAPE, "dfs_select_mask: M_v=%d exceeds 16128 (one score row and a histogram must fit in 64 KB of LDS)", s.M_v);
  const int k_base = dfs_keep_count(sparsity, s.M_v);
  if (K_max < k_base + s.M_x)
    return fail(DFS_ESHAPE, "dfs_select_mask: K_max=%d is below the %d kept blocks per row", K_max, k_base + s.M_x);
  const size_t lds = size_t(s.M_v) * sizeof(uint32_t);            // the mass count keeps one key per column
  const size_t lds_sel = lds + 256 * sizeof(uint32_t);           // the selection adds its byte histogram
  dim3 rows(unsigned(s.M), unsigned(g->heads));
  if (mode == DFS_SELECT_TOPK) {
    select_kernel<<<rows, 64, lds_sel, st>>>(score, s.M_v, s.M_x, k_base, nullptr, nullptr, 0, mask, kv_idx, kv_cnt, K_max, k_head);
  } else {
    if (!(mass > 0.0 && mass <= 1.0)) return fail(DFS_EINVAL, "dfs_select_mask: mass %g is outside (0,1]", mass);
    int32_t* k_row = static_cast<int32_t*>(ws);
    int32_t* k_used = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + align256(size_t(g->heads) * s.M_v * sizeof(int32_t)));
    int k_cap = K_max - s.M_x;
    if (k_cap > s.M_v) k_cap = s.M_v;
    mass_count_kernel<<<dim3(unsigned(s.M_v), unsigned(g->heads)), 64, lds, st>>>(score, s.M_v, mass, k_row);
    if (mode == DFS_SELECT_MASS_HEAD) {
      head_count_kernel<<<dim3(unsigned(g->heads)), 256, 0, st>>>(k_row, s.M_v, k_base, k_cap, k_used, k_head);
      select_kernel<<<rows, 64, lds_sel, st>>>(score, s.M_v, s.M_x, 0, k_used, nullptr, 0, mask, kv_idx, kv_cnt, K_max, nullptr);
    } else {
      select_kernel<<<rows, 64, lds_sel, st>>>(score, s.M_v, s.M_x, k_base, nullptr, k_row, k_cap, mask, kv_idx, kv_cnt, K_max, nullptr);
    }
  }
  return launch_status("dfs_select_mask");
}

// Device address of `scratch` on the current device, resolved on the first call per device and kept.
static int static_scratch(void** out) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static void* addr[MAX_DEV] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(DFS_EHIP, "dfs_select_mask_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= MAX_DEV) return fail(DFS_EHIP, "dfs_select_mask_static: device ordinal %d is outside [0,%d)", dev, MAX_DEV);
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(DFS_EHIP, "dfs_select_mask_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    addr[dev] = p;
  }
  *out = addr[dev];
  return DFS_OK;
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_select_mask_static(const dfs_geom* g, const float* score, int mode, double sparsity, double mass, uint8_t* mask,
                                      int32_t* kv_idx, int32_t* kv_cnt, int32_t K_max, int32_t* k_head, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (!score || !kv_idx || !kv_cnt) return fail(DFS_EINVAL, "dfs_select_mask_static: NULL argument");
  if (misaligned(4, {score, kv_idx, kv_cnt, k_head})) return fail(DFS_EINVAL, "dfs_select_mask_static: score, list and count arrays must be 4-byte aligned");
  const size_t need = ws_select_mask(g, s);
  if (need > STATIC_SCRATCH_BYTES)
    return fail(DFS_EWORKSPACE, "dfs_select_mask_static: heads x M_v = %d x %d needs %zu bytes of scratch, the built-in buffer holds %zu; "
                                "use dfs_select_mask with a workspace", g->heads, s.M_v, need, STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  return run_select_mask(g, s, score, mode, sparsity, mass, mask, kv_idx, kv_cnt, K_max, k_head, ws, as_stream(stream));
}

extern "C" int dfs_select_mask(const dfs_geom* g, const float* score, int mode, double sparsity, double mass, uint8_t* mask,
                               int32_t* kv_idx, int32_t* kv_cnt, int32_t K_max, int32_t* k_head, void* ws, size_t ws_bytes,
                               void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (!score || !kv_idx || !kv_cnt) return fail(DFS_EINVAL, "dfs_select_mask: NULL argument");
  if (misaligned(4, {score, kv_idx, kv_cnt, k_head})) return fail(DFS_EINVAL, "dfs_select_mask: score, list and count arrays must be 4-byte aligned");
  const size_t need = ws_select_mask(g, s);
  if ((mode == DFS_SELECT_MASS_HEAD || mode == DFS_SELECT_MASS_ROW) && (!ws || (uintptr_t(ws) & 255) || ws_bytes < need))
    return fail(DFS_EWORKSPACE, "dfs_select_mask: workspace of %zu bytes needed (256-byte aligned), got %zu", need, ws_bytes);
  return run_select_mask(g, s, score, mode, sparsity, mass, mask, kv_idx, kv_cnt, K_max, k_head, ws, as_stream(stream));
}
