// Host side of the C ABI: geometry checks, error state, workspace sizes, and the one-call
// form of the paper's Algorithm 1.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include "common.h"

namespace dfs {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(DFS_EHIP, "%s: %s", what, hipGetErrorString(e));
  return DFS_OK;
}

int check_geom(const dfs_geom* g, dfs_sizes* s) {
  if (!g) return fail(DFS_EINVAL, "geometry pointer is NULL");
  if (g->T < 1 || g->H < 1 || g->W < 1 || g->T > 512 || g->H > 512 || g->W > 512)
    return fail(DFS_ESHAPE, "grid %dx%dx%d: each axis must be in [1,512]", g->T, g->H, g->W);
  if (g->n_text < 0) return fail(DFS_ESHAPE, "n_text=%d is negative", g->n_text);
  if (g->heads < 1) return fail(DFS_ESHAPE, "heads=%d must be positive", g->heads);
  if (g->d != 64 && g->d != 128) return fail(DFS_ESHAPE, "d=%d: head dimension must be 64 or 128", g->d);
  if (g->B != 64 && g->B != 128) return fail(DFS_ESHAPE, "B=%d: block size must be 64 or 128", g->B);
  if (g->Bs < 1 || g->B % g->Bs != 0) return fail(DFS_ESHAPE, "Bs=%d must divide B=%d", g->Bs, g->B);
  int r = g->B / g->Bs;
  if (r != 1 && r != 2 && r != 4 && r != 8) return fail(DFS_ESHAPE, "B/Bs=%d must be 1, 2, 4 or 8", r);
  int64_t N_v = int64_t(g->T) * g->H * g->W;
  int64_t N = N_v + g->n_text;
  int64_t M_v = (N_v + g->B - 1) / g->B, M_x = (int64_t(g->n_text) + g->B - 1) / g->B;
  if (M_v + M_x > 65536) return fail(DFS_ESHAPE, "M=%lld blocks exceeds 65536", (long long)(M_v + M_x));
  if ((M_v + M_x) * g->B * int64_t(g->heads) >= (int64_t(1) << 40))
    return fail(DFS_ESHAPE, "heads*N_pad too large");
  int mx = g->T > g->H ? g->T : g->H;
  if (g->W > mx) mx = g->W;
  int bits = 1;
  while ((1 << bits) < mx) ++bits;
  if (s) {
    s->N_v = N_v; s->N = N; s->M_v = int32_t(M_v); s->M_x = int32_t(M_x); s->M = int32_t(M_v + M_x);
    s->N_pad = (M_v + M_x) * g->B; s->r = r; s->M_s = int32_t(M_v * r); s->bits = bits;
  }
  return DFS_OK;
}

struct FwdLayout { size_t qp, kp, vp, op, score, sub, total; };

static FwdLayout forward_layout(const dfs_geom* g, const dfs_sizes& s, int dtype) {
  FwdLayout L;
  size_t t = align256(size_t(g->heads) * s.N_pad * g->d * elem_size(dtype));
  size_t off = 0;
  L.qp = off; off += t;
  L.kp = off; off += t;
  L.vp = off; off += t;
  L.op = off; off += t;
  L.score = off; off += align256(size_t(g->heads) * s.M_v * s.M_v * sizeof(float));
  L.sub = off;
  size_t a = ws_block_score(g, s), b = ws_select_mask(g, s);
  off += a > b ? a : b;
  L.total = off;
  return L;
}

}  // namespace dfs

using namespace dfs;

extern "C" {

const char* dfs_last_error(void) { return g_err; }

int dfs_geom_sizes(const dfs_geom* g, dfs_sizes* out) {
  if (!out) return fail(DFS_EINVAL, "sizes pointer is NULL");
  return check_geom(g, out);
}

int32_t dfs_keep_count(double sparsity, int32_t M_v) {
  if (M_v < 1 || !(sparsity >= 0.0 && sparsity <= 1.0)) return 0;
  double k = ceil((1.0 - sparsity) * double(M_v) - 1e-6);
  if (k < 1.0) k = 1.0;
  if (k > double(M_v)) k = double(M_v);
  return int32_t(k);
}

size_t dfs_workspace_bytes(const dfs_geom* g, int kind) {
  dfs_sizes s;
  if (check_geom(g, &s) != DFS_OK) return 0;
  switch (kind) {
    case DFS_WS_HILBERT_PERM: return ws_hilbert(g, s);
    case DFS_WS_BLOCK_SCORE: return ws_block_score(g, s);
    case DFS_WS_SELECT_MASK: return ws_select_mask(g, s);
    case DFS_WS_FORWARD: return forward_layout(g, s, DFS_F32).total;
    case DFS_WS_FORWARD_BF16: return forward_layout(g, s, DFS_BF16).total;
    default: fail(DFS_EINVAL, "unknown workspace kind %d", kind); return 0;
  }
}

int dfs_forward(const dfs_geom* g, int dtype, const void* q, const void* k, const void* v,
                const int32_t* perm_pad, const int32_t* inv, int refresh, int mode, double sparsity,
                double mass, dfs_mask_state* st, float scale, void* o, void* ws, size_t ws_bytes,
                void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_F32 && dtype != DFS_BF16) return fail(DFS_EDTYPE, "dtype %d is not DFS_F32 or DFS_BF16", dtype);
  if (!q || !k || !v || !o || !perm_pad || !inv || !st) return fail(DFS_EINVAL, "dfs_forward: NULL argument");
  if (misaligned(16, {q, k, v, o}) || misaligned(4, {perm_pad, inv, st->kv_idx, st->kv_cnt, st->k_head}))
    return fail(DFS_EINVAL, "dfs_forward: tensors must be 16-byte aligned, index arrays 4-byte aligned");
  if (!st->kv_idx || !st->kv_cnt) return fail(DFS_EINVAL, "dfs_forward: mask state has no kv_idx/kv_cnt");
  FwdLayout L = forward_layout(g, s, dtype);
  if (!ws || (uintptr_t(ws) & 255) || ws_bytes < L.total)
    return fail(DFS_EWORKSPACE, "dfs_forward: workspace of %zu bytes needed (256-byte aligned), got %zu", L.total, ws_bytes);
  char* base = static_cast<char*>(ws);
  hipStream_t hs = as_stream(stream);
  // bf16: Q is gathered where it is consumed (pooling, attention) and O is scattered by the attention kernel,
  // so only K and V take a reorder pass.  fp32 (small problems): every tensor is reordered.
  const bool fused = dtype == DFS_BF16;
  const int32_t* index = fused ? perm_pad : nullptr;
  const void* q_in = fused ? q : base + L.qp;
  void* o_out = fused ? o : base + L.op;
  if (!fused && (rc = run_permute(g, s, dtype, q, perm_pad, base + L.qp, hs))) return rc;
  // On a refresh step of the bf16 path the pooling kernel reorders K on the way (it reads K in source order
  // and writes K'), which spares that reorder pass too.
  const bool k_in_pool = fused && refresh;
  if (!k_in_pool && (rc = run_permute(g, s, dtype, k, perm_pad, base + L.kp, hs))) return rc;
  if ((rc = run_permute(g, s, dtype, v, perm_pad, base + L.vp, hs))) return rc;
  if (refresh) {
    float* score = reinterpret_cast<float*>(base + L.score);
    if ((rc = run_block_score(g, s, dtype, q_in, k_in_pool ? k : static_cast<const void*>(base + L.kp), score, base + L.sub, index,
                              k_in_pool ? base + L.kp : nullptr, hs)))
      return rc;
    if ((rc = run_select_mask(g, s, score, mode, sparsity, mass, st->mask, st->kv_idx, st->kv_cnt, st->K_max,
                              st->k_head, base + L.sub, hs)))
      return rc;
  }
  if ((rc = run_sparse_attn(g, s, dtype, q_in, base + L.kp, base + L.vp, st->kv_idx, st->kv_cnt, st->K_max, scale, o_out,
                            nullptr, index, hs)))
    return rc;
  if (!fused) return run_unperm(g, s, dtype, base + L.op, inv, o, hs);
  return DFS_OK;
}

int dfs_schedule(int32_t total_steps, int32_t t, int32_t delta, double cached_keep, int32_t* dense, int32_t* refresh,
                 double* sparsity) {
  if (!dense || !refresh || !sparsity) return fail(DFS_EINVAL, "dfs_schedule: NULL output");
  if (total_steps < 1 || t < 0 || t >= total_steps || delta < 1)
    return fail(DFS_EINVAL, "dfs_schedule: need 0 <= t < total_steps and delta >= 1 (got t=%d, total=%d, delta=%d)", t, total_steps, delta);
  int quarter = int(floor(double(t) / (0.25 * double(total_steps)) + 1e-9));
  if (quarter > 3) quarter = 3;
  if (quarter == 0) {
    *dense = 1; *refresh = 0; *sparsity = 0.0;
    return DFS_OK;
  }
  const double keep = 0.3 - 0.1 * double(quarter - 1);
  *dense = 0;
  *sparsity = 1.0 - keep;
  *refresh = (t % delta == 0) || cached_keep < 0.0 || fabs(cached_keep - keep) > 1e-12;
  return DFS_OK;
}

}  // extern "C"
