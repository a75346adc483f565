// Measurement probes, not part of the method: what the chip sustains on bare matrix-instruction chains and
// on a plain copy, to set beside the nominal peaks the roofline fractions are quoted against.
#include "common.h"

namespace dfs {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Four independent accumulator chains of v_mfma_f32_32x32x16_bf16 per wave, nothing else in the loop.
// counters (optional): [0] += shader-clock cycles, [1] += 100 MHz ticks of work-group 0's lifetime.
__global__ void __launch_bounds__(256) mfma_chain_kernel(float* __restrict__ sink, unsigned long long* __restrict__ counters,
                                                         int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float(threadIdx.x & 7) * 0.125f + i); b[i] = (__bf16)(0.25f * i); }
  f32x16 c0 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 c1 = c0, c2 = c0, c3 = c0;
  const unsigned long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  if (counters && blockIdx.x == 0 && threadIdx.x == 0) {
    atomicAdd(&counters[0], clock64() - t0);
    atomicAdd(&counters[1], wall_clock64() - w0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// 16 bytes per lane, grid-stride.
__global__ void __launch_bounds__(256) copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n16; i += size_t(gridDim.x) * 256) dst[i] = src[i];
}

// Read-only traffic of the shape the attention kernel's tile loads have: every work-group reads `pieces_per_wg` 64 KB
// pieces of the region at seeded pseudo-random piece indices (non-temporal 16-byte loads) and does nothing else.
// The checksum keeps the loads alive; sink[0] is written only if it takes one particular value.
__global__ void __launch_bounds__(256) read_pieces_kernel(const u32x4* __restrict__ src, unsigned long long pieces, int pieces_per_wg,
                                                          unsigned int* __restrict__ sink) {
  unsigned int acc = 0, seed = blockIdx.x * 2654435761u + 12345u;
  for (int i = 0; i < pieces_per_wg; ++i) {
    seed = seed * 1664525u + 1013904223u;
    const unsigned long long piece = ((unsigned long long)(seed >> 8) * pieces) >> 24;   // < pieces
    const u32x4* p = src + piece * 4096;
#pragma unroll
    for (int j = 0; j < 16; ++j) {                                                          // 256 threads x 16 B x 16
      const u32x4 v = __builtin_nontemporal_load(p + j * 256 + threadIdx.x);
      acc += v[0] ^ v[1] ^ v[2] ^ v[3];
    }
  }
  if (acc == 0x12345678u) sink[0] = acc;
}

}  // namespace dfs

using namespace dfs;

extern "C" int dfs_probe_mfma(int32_t work_groups, int32_t iters, float* sink, uint64_t* counters, void* stream) {
  if (work_groups < 1 || work_groups > 65535 || iters < 1) return fail(DFS_EINVAL, "dfs_probe_mfma: need 1 <= work_groups <= 65535 and iters >= 1");
  if (!sink) return fail(DFS_EINVAL, "dfs_probe_mfma: NULL sink");
  if (misaligned(4, {sink}) || misaligned(8, {counters})) return fail(DFS_EINVAL, "dfs_probe_mfma: sink must be 4-byte, counters 8-byte aligned");
  mfma_chain_kernel<<<unsigned(work_groups), 256, 0, as_stream(stream)>>>(sink, reinterpret_cast<unsigned long long*>(counters), iters);
  return launch_status("dfs_probe_mfma");
}

extern "C" int dfs_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return fail(DFS_EINVAL, "dfs_probe_copy: NULL argument");
  if (bytes % 16 || misaligned(16, {src, dst})) return fail(DFS_EINVAL, "dfs_probe_copy: pointers and size must be multiples of 16 bytes");
  copy_kernel<<<8192, 256, 0, as_stream(stream)>>>(static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
  return launch_status("dfs_probe_copy");
}

extern "C" int dfs_probe_read(const void* src, size_t bytes, int32_t work_groups, int32_t pieces_per_wg, uint32_t* sink, void* stream) {
  if (!src || !sink) return fail(DFS_EINVAL, "dfs_probe_read: NULL argument");
  if (bytes < 65536 || bytes % 65536 || misaligned(16, {src}) || misaligned(4, {sink}))
    return fail(DFS_EINVAL, "dfs_probe_read: the region must be a multiple of 64 KB and 16-byte aligned, sink 4-byte aligned");
  if (work_groups < 1 || work_groups > 65535 || pieces_per_wg < 1) return fail(DFS_EINVAL, "dfs_probe_read: need 1 <= work_groups <= 65535 and pieces_per_wg >= 1");
  if (bytes / 65536 > (1ull << 24)) return fail(DFS_EINVAL, "dfs_probe_read: region above 1 TiB");
  read_pieces_kernel<<<unsigned(work_groups), 256, 0, as_stream(stream)>>>(static_cast<const u32x4*>(src), bytes / 65536, pieces_per_wg, sink);
  return launch_status("dfs_probe_read");
}
