// Internal helpers shared by the HIP translation units of libdfsattn (not part of the ABI).
#pragma once
#include <initializer_list>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dfsattn.h"

namespace dfs {

// Records `msg` as the calling thread's last error and returns `code`.
int fail(int code, const char* fmt, ...);
// Validates a geometry (sets the error on failure) and fills the derived sizes.
int check_geom(const dfs_geom* g, dfs_sizes* s);
// Turns the error state left by a kernel launch into a status code.
int launch_status(const char* what);

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
// Tensor rows move 16 bytes at a time, so every Q/K/V/O tensor must start on a 16-byte boundary
// (index, count and fp32 arrays on a 4-byte boundary).  True if any of the pointers does not.
inline bool misaligned(size_t a, std::initializer_list<const void*> ps) {
  for (const void* p : ps)
    if (reinterpret_cast<uintptr_t>(p) & (a - 1)) return true;
  return false;
}
inline int elem_size(int dtype) { return dtype == DFS_BF16 ? 2 : 4; }

// Stage entry points without argument checks, used by dfs_forward after it has validated once.
int run_permute(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* x, const int32_t* perm_pad,
                void* x_perm, hipStream_t st);
// q_index (may be NULL): the permutation; Q is then read in source order and gathered while pooling.
int run_block_score(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q_perm, const void* k_perm,
                    float* score, void* ws, const int32_t* q_index, void* k_out, hipStream_t st);
int run_select_mask(const dfs_geom* g, const dfs_sizes& s, const float* score, int mode, double sparsity,
                    double mass, uint8_t* mask, int32_t* kv_idx, int32_t* kv_cnt, int32_t K_max,
                    int32_t* k_head, void* ws, hipStream_t st);
int run_sparse_attn(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q, const void* k, const void* v,
                    const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale, void* o, float* lse,
                    const int32_t* row_index, hipStream_t st);   // row_index (may be NULL, bf16 only): Q and O in source order
int run_unperm(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* o_perm, const int32_t* inv, void* o,
               hipStream_t st);
size_t ws_block_score(const dfs_geom* g, const dfs_sizes& s);
size_t ws_select_mask(const dfs_geom* g, const dfs_sizes& s);
size_t ws_hilbert(const dfs_geom* g, const dfs_sizes& s);

// bf16 <-> fp32 on raw bits (round to nearest even on the way down)
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

}  // namespace dfs
