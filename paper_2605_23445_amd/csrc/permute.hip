// Row gathers that apply the token permutation and its inverse (Algorithm 1 steps 1 and 3).
// Pure data movement, bound by HBM: every lane moves 16 bytes, the lanes of a row are adjacent,
// writes are fully sequential and reads are whole rows (128-512 bytes) whose sources are near
// each other because consecutive Hilbert positions are neighbouring cells.
#include "common.h"

namespace dfs {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// dst[h, p, :] = idx[p] >= 0 ? src[h, idx[p], :] : 0     rows of `row16` 16-byte chunks
// One thread block covers ROWS consecutive destination rows of one head.
template <int ROW16>
__global__ void __launch_bounds__(256) gather_rows_kernel(const u32x4* __restrict__ src, const int32_t* __restrict__ idx,
                                                          u32x4* __restrict__ dst, int64_t n_dst, int64_t n_src) {
  constexpr int ROWS_PER_PASS = 256 / ROW16;
  constexpr int PASSES = 4;
  const int head = blockIdx.y;
  const int c = threadIdx.x % ROW16;
  const int rl = threadIdx.x / ROW16;
  const int64_t row0 = int64_t(blockIdx.x) * (ROWS_PER_PASS * PASSES);
  const u32x4* s = src + int64_t(head) * n_src * ROW16;
  u32x4* d = dst + int64_t(head) * n_dst * ROW16;
  u32x4 val[PASSES];
  int64_t rows[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int64_t row = row0 + p * ROWS_PER_PASS + rl;
    rows[p] = row;
    int32_t from = row < n_dst ? idx[row] : -1;
    val[p] = u32x4{0u, 0u, 0u, 0u};
    if (from >= 0 && from < n_src) val[p] = __builtin_nontemporal_load(&s[int64_t(from) * ROW16 + c]);
  }
#pragma unroll
  for (int p = 0; p < PASSES; ++p)
    if (rows[p] < n_dst) __builtin_nontemporal_store(val[p], &d[rows[p] * ROW16 + c]);
}

static int launch_gather(int row_bytes, const void* src, const int32_t* idx, void* dst, int64_t n_dst, int64_t n_src,
                         int heads, hipStream_t st) {
  const int row16 = row_bytes / 16;
  const int rows_per_block = (256 / row16) * 4;
  dim3 grid(unsigned((n_dst + rows_per_block - 1) / rows_per_block), unsigned(heads));
  const u32x4* s = static_cast<const u32x4*>(src);
  u32x4* d = static_cast<u32x4*>(dst);
  switch (row16) {
    case 8: gather_rows_kernel<8><<<grid, 256, 0, st>>>(s, idx, d, n_dst, n_src); break;
    case 16: gather_rows_kernel<16><<<grid, 256, 0, st>>>(s, idx, d, n_dst, n_src); break;
    case 32: gather_rows_kernel<32><<<grid, 256, 0, st>>>(s, idx, d, n_dst, n_src); break;
    default: return fail(DFS_ESHAPE, "row of %d bytes is not supported", row_bytes);
  }
  return DFS_OK;
}

int run_permute(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* x, const int32_t* perm_pad, void* x_perm,
                hipStream_t st) {
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  int rc = launch_gather(g->d * elem_size(dtype), x, perm_pad, x_perm, s.N_pad, s.N, g->heads, st);
  return rc ? rc : launch_status("dfs_permute");
}

int run_unperm(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* o_perm, const int32_t* inv, void* o,
               hipStream_t st) {
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  int rc = launch_gather(g->d * elem_size(dtype), o_perm, inv, o, s.N, s.N_pad, g->heads, st);
  return rc ? rc : launch_status("dfs_unperm");
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_permute(const dfs_geom* g, int dtype, const void* x, const int32_t* perm_pad, void* x_perm, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_F32 && dtype != DFS_BF16) return fail(DFS_EDTYPE, "dtype %d is not DFS_F32 or DFS_BF16", dtype);
  if (!x || !perm_pad || !x_perm) return fail(DFS_EINVAL, "dfs_permute: NULL argument");
  if (misaligned(16, {x, x_perm}) || misaligned(4, {perm_pad})) return fail(DFS_EINVAL, "dfs_permute: tensors must be 16-byte aligned, the index array 4-byte aligned");
  return run_permute(g, s, dtype, x, perm_pad, x_perm, as_stream(stream));
}

extern "C" int dfs_unperm(const dfs_geom* g, int dtype, const void* o_perm, const int32_t* inv, void* o, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_F32 && dtype != DFS_BF16) return fail(DFS_EDTYPE, "dtype %d is not DFS_F32 or DFS_BF16", dtype);
  if (!o_perm || !inv || !o) return fail(DFS_EINVAL, "dfs_unperm: NULL argument");
  if (misaligned(16, {o_perm, o}) || misaligned(4, {inv})) return fail(DFS_EINVAL, "dfs_unperm: tensors must be 16-byte aligned, the index array 4-byte aligned");
  return run_unperm(g, s, dtype, o_perm, inv, o, as_stream(stream));
}
