// Attention recall (paper Eq. 3) from two log-sum-exp arrays: the share of a query row's attention
// mass that the kept keys hold is exp(lse under the mask - lse with every block kept); the recall of
// a head is the mean of that share over its real query rows.
#include "common.h"

namespace dfs {

// One work-group per head.  Fixed assignment of rows to threads and a fixed reduction tree: reruns
// give the same bits.
__global__ void __launch_bounds__(256) recall_kernel(const float* __restrict__ lse_sparse, const float* __restrict__ lse_dense,
                                                     float* __restrict__ recall, int64_t N_pad, int64_t N_v, int64_t text_base,
                                                     int n_text) {
  __shared__ double part[4];
  const int head = blockIdx.x;
  const float* a = lse_sparse + int64_t(head) * N_pad;
  const float* b = lse_dense + int64_t(head) * N_pad;
  double acc = 0.0;
  for (int64_t p = threadIdx.x; p < N_pad; p += 256) {
    const bool real = p < N_v || (p >= text_base && p - text_base < n_text);
    if (real) {
      const float d = a[p] - b[p];                 // <= 0 up to rounding; -inf for a row that keeps nothing
      acc += double(d == d ? __expf(d) : 0.f);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const int lo = __shfl_xor(__double2loint(acc), off, 64), hi = __shfl_xor(__double2hiint(acc), off, 64);
    acc += __hiloint2double(hi, lo);
  }
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) recall[head] = float((part[0] + part[1] + part[2] + part[3]) / double(N_v + n_text));
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_recall(const dfs_geom* g, const float* lse_sparse, const float* lse_dense, float* recall, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (!lse_sparse || !lse_dense || !recall) return fail(DFS_EINVAL, "dfs_recall: NULL argument");
  if (misaligned(4, {lse_sparse, lse_dense, recall})) return fail(DFS_EINVAL, "dfs_recall: fp32 arrays must be 4-byte aligned");
  if (g->heads > 65535) return fail(DFS_ESHAPE, "heads=%d exceeds 65535", g->heads);
  recall_kernel<<<dim3(unsigned(g->heads)), 256, 0, as_stream(stream)>>>(lse_sparse, lse_dense, recall, s.N_pad, s.N_v,
                                                                        int64_t(s.M_v) * g->B, g->n_text);
  return launch_status("dfs_recall");
}
