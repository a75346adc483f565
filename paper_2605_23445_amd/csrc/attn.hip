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
#include <type_traits>

#include "common.h"

namespace dfs {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int KN = 64;   // key rows per LDS tile

__device__ __forceinline__ int block_real_rows(int blk, int B, int M_v, int64_t N_v, int n_text) {
  int64_t real = blk < M_v ? N_v - int64_t(blk) * B : int64_t(n_text) - int64_t(blk - M_v) * B;
  return real >= B ? B : (real <= 0 ? 0 : int(real));
}

// XOR swizzles of the 16-byte chunks inside a tile row.  Tiles are stored without padding (the
// direct-to-LDS load writes 64 consecutive chunks per wave instruction); the swizzle, applied on the
// global side of the load and again on every LDS read, spreads the rows a wave reads at once over
// all banks.  K is read one row per lane (16 B each), V four rows x 64 B per half-wave pass.
template <int CH> __device__ __forceinline__ int swz_k(int row) { return (row / (16 / CH)) % CH; }
template <int CH> __device__ __forceinline__ int swz_v(int row) { return 4 * ((row / (16 / CH)) % (CH / 4)); }

constexpr int swz_period(int step, int mod) {    // smallest P with (P * step) % mod == 0
  int p = 1;
  while ((p * step) % mod != 0) ++p;
  return p;
}

// Maxima as single instructions.  (fmaxf on raw matrix-instruction results makes the compiler add a
// canonicalising v_max per input.)  The inputs are logits or -inf, never NaN.  The instructions read
// results of matrix instructions issued at least a whole softmax slice plus a stage prologue earlier,
// far beyond the wait states such a read needs.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float max2(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// QT = 32-row query tiles per wave.  With QT = 2 every K / V^T fragment read from LDS feeds two
// matrix instructions, which halves the LDS bytes per matrix instruction, but at d = 128 the
// accumulators then need the whole register file, i.e. one wave per SIMD.  Measured: the lone wave runs
// at a higher clock (2.1 against 1.8 GHz, it draws less power) but keeps the matrix cores busy only
// 43 % of the cycles against 57 % for two waves: a wave issues in order, about one instruction per five
// cycles, and one wave's stream of ~9 instructions per matrix instruction cannot fill the pipe alone.
// Net 960 against 1070 TFLOP/s on cache-resident keys, so QT = 1 is what is launched.
//
// XLSE: the caller wants the log-sum-exp.  The normaliser of O sums the probabilities as rounded to bf16
// (see `pack` below), which is right for O but leaves ln(sum) off by up to bf16's unit roundoff 2^-8; with
// XLSE a second running sum of the unrounded fp32 probabilities is kept for the log-sum-exp alone.
//
// Waves per SIMD: two at d = 128 (about 250 registers each).  At d = 64 the kernel needs about 160 registers, so
// three waves fit (measured 36 -> 43 % of the matrix cycles, +8 % throughput on the 17 550- and 75 600-token
// shapes); the variants that would have to spill for that (64-row blocks, log-sum-exp output) stay at two.
template <int D, int QT, int BM, bool XLSE>
constexpr int attn_waves() { return D == 64 && QT == 1 && BM == 128 && !XLSE ? 3 : 2 / QT; }
template <int D, int BM, int QT, bool XLSE>
__global__ void __launch_bounds__(BM * 2 / QT)
__attribute__((amdgpu_waves_per_eu(attn_waves<D, QT, BM, XLSE>(), attn_waves<D, QT, BM, XLSE>())))
attn_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                 const int32_t* __restrict__ kv_idx, const int32_t* __restrict__ kv_cnt, int K_max, uint16_t* __restrict__ o,
                 float* __restrict__ lse, const int32_t* __restrict__ row_index, int64_t N_src, int64_t N_pad, int64_t N_v, int n_text,
                 int M_v, int M, int total_wg, int wg_per_xcd, int mapping, float scale, unsigned long long* __restrict__ clock_probe) {
  constexpr int NW = BM / (32 * QT);               // waves: one per 32 QT query rows
  constexpr int CH = D / 8;                        // 16-byte chunks per row
  constexpr int TILE = KN * D;                     // elements per tile
  constexpr int LPW = KN * CH / (64 * NW);         // load instructions per wave and tile
  constexpr int RJ = NW * 64 / CH;                 // tile rows between two load instructions of a wave
  constexpr int STEPS = BM / KN;                   // tiles per key block
  constexpr int NF = D / 8;                        // operand fragments per stage: D/16 of V^T, D/16 of K
  constexpr int SLOTS = NF * QT;                   // matrix instructions per stage
  constexpr int ESL = 12;                          // slices the sixteen exponentials of a query tile are spread over
  constexpr int SL = 5 + ESL;                      // softmax slices per query tile: 4 for the maximum, ESL, 1 to close
  constexpr int SLICES = SL * QT;                  // softmax slices per stage
  constexpr int STAGE_LEN = SLOTS > SLICES ? SLOTS : SLICES;
  constexpr float TAU = 8.f;                       // rescale only when the row maximum grows by > 2^TAU
  // Two K and two V tile buffers (tile t lives in the pair of parity t & 1).
  __shared__ __attribute__((aligned(16))) uint16_t sK0[TILE];
  __shared__ __attribute__((aligned(16))) uint16_t sK1[TILE];
  __shared__ __attribute__((aligned(16))) uint16_t sV0[TILE];
  __shared__ __attribute__((aligned(16))) uint16_t sV1[TILE];

  // Work-group to (head, query block).  Ids are dealt round-robin to the 8 XCDs, so id % 8 names the XCD
  // and id / 8 the order inside it.
  //   mapping 2 (long sequences): every XCD takes its own eighth of the query blocks of head 0, then of
  //     head 1, ...  All XCDs are on the same head at the same time, so the key/value working set of the
  //     chip is one or two heads and stays in the memory-side cache, while the blocks that meet in one
  //     L2 are neighbours on the curve, which share key blocks.  The dense text blocks of all heads, the
  //     longest work-groups, come first.
  //   mapping 1 (an eighth of a head would not fill an XCD): each XCD walks whole heads of its own,
  //     query blocks last-first so that the text blocks of a head start first.
  //   mapping 0: ids in plain order.
  int head, u;
  if (mapping == 2) {
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int M_x = M - M_v, n_heads = total_wg / M;
    const int text_slots = (n_heads * M_x + 7) / 8;
    if (slot < text_slots) {
      const int id = slot * 8 + xcd;
      if (id >= n_heads * M_x) return;
      head = id / M_x;
      u = M_v + id % M_x;
    } else {
      const int C = (M_v + 7) / 8, s2 = slot - text_slots;
      head = s2 / C;
      u = xcd * C + s2 % C;
      if (head >= n_heads || u >= M_v) return;
    }
  } else {
    const int logical = mapping ? (blockIdx.x % 8) * wg_per_xcd + blockIdx.x / 8 : blockIdx.x;
    if (logical >= total_wg) return;
    head = logical / M;
    u = M - 1 - logical % M;
  }

  // diagnostic: shader-clock cycles and constant-rate (100 MHz) ticks this work-group lives for
  const unsigned long long probe_c0 = clock_probe ? clock64() : 0, probe_w0 = clock_probe ? wall_clock64() : 0;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int cnt_in = kv_cnt[int64_t(head) * M + u];
  const bool dense = cnt_in >= M;
  const int cnt = dense ? M : (cnt_in < 0 ? 0 : (cnt_in > K_max ? K_max : cnt_in));
  const int32_t* idx = kv_idx + (int64_t(head) * M + u) * K_max;
  const int64_t head_off = int64_t(head) * N_pad * D;
  const uint16_t* kh = k + head_off;
  const uint16_t* vh = v + head_off;
  const int64_t q_row0 = int64_t(u) * BM + wave * (32 * QT) + n;      // query tile a adds 32 a

  // Where this lane's query rows live.  With row_index (the permutation) Q is read from, and O written to,
  // the tensors in source order, which spares the reorder passes of Q and O; -1 marks a pad row.
  int64_t io_row[QT];
#pragma unroll
  for (int a = 0; a < QT; ++a) {
    const int64_t pos = q_row0 + 32 * a;
    io_row[a] = row_index ? int64_t(row_index[pos]) : pos;
    if (row_index && io_row[a] >= N_src) io_row[a] = -1;
  }
  const int64_t io_off = int64_t(head) * (row_index ? N_src : N_pad) * D;

  // Q rows as the B operand of S^T = K Q^T: lane (n, h) holds Q[row][16 kk + 8 h .. + 7]
  bf16x8 qf[QT][D / 16];
#pragma unroll
  for (int a = 0; a < QT; ++a) {
    const u32x4* qp = reinterpret_cast<const u32x4*>(q + io_off + (io_row[a] < 0 ? 0 : io_row[a]) * D);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
      qf[a][kk] = __builtin_bit_cast(bf16x8, io_row[a] < 0 ? u32x4{0u, 0u, 0u, 0u} : qp[2 * kk + h]);
  }

  f32x16 oacc[QT][D / 32];
#pragma unroll
  for (int a = 0; a < QT; ++a)
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[a][dt][i] = 0.f;
  float m_run[QT], l_run[QT], x_run[QT];           // x_run: unrounded normaliser (XLSE only)
  // m_run is the reference maximum in the base-2 exponent's units (logit x c2).  It starts at a large
  // finite negative value instead of -inf, so that a row that has only met pad keys (all logits -inf)
  // needs no special case: its differences stay finite and its probabilities are exp2(-inf) = 0.
  constexpr float M_START = -1.0e30f;
#pragma unroll
  for (int a = 0; a < QT; ++a) { m_run[a] = M_START; l_run[a] = 0.f; x_run[a] = 0.f; }
  const float c2 = scale * 1.4426950408889634f;     // softmax in base 2

  // Tile loads, global memory straight into LDS: instruction j of this wave fills the 64 consecutive
  // 16-byte chunks (j NW + wave) 64 + lane of the tile buffer; the chunk swizzle is applied on the
  // global side.  The swizzle repeats every PK (PV) instructions, so that few per-lane offsets serve all.
  constexpr int PK = swz_period(RJ / (16 / CH) > 0 ? RJ / (16 / CH) : 1, CH);
  constexpr int PV = swz_period(RJ / (16 / CH) > 0 ? RJ / (16 / CH) : 1, CH / 4);
  static_assert(RJ % (16 / CH) == 0 && LPW % PK == 0 && LPW % PV == 0, "tile load pattern");
  const int n_tiles = cnt * STEPS;
  auto tile_block = [&](int tile) {
    int blk = dense ? tile / STEPS : idx[tile / STEPS];
    return unsigned(blk) < unsigned(M) ? blk : 0;     // a corrupt list must not read out of bounds
  };
  auto lane_off = [&](int j, bool is_v) {             // byte offset inside the tile of the chunk this lane fetches
    const int p = (j * NW + wave) * 64 + lane;
    const int row = p / CH, pc = p % CH;
    return uint32_t(2 * (row * D + ((pc ^ (is_v ? swz_v<CH>(row) : swz_k<CH>(row))) * 8)));
  };
  uint32_t k_off[PK], v_off[PV];
#pragma unroll
  for (int j = 0; j < PK; ++j) k_off[j] = lane_off(j, false);
#pragma unroll
  for (int j = 0; j < PV; ++j) v_off[j] = lane_off(j, true);
  // The load is issued from an asm statement so that it stays outside the compiler's wait-count
  // bookkeeping: the compiler cannot tell that reads of one tile buffer are independent of loads in
  // flight into another and would wait for every outstanding load before each LDS read.  The waits
  // that are needed are the explicit vmcnt(0) + barrier pairs in the loop below.  (Loads retire in
  // order, so the compiler's own counts for its few other memory operations stay conservative.)
  // LDS addresses of this wave's first chunk in each tile buffer, as scalars, once (taken from a vector register
  // inside the loop they cost a vector-to-scalar hand-over per tile)
  auto lds_base = [&](uint16_t* buf) {
    return __builtin_amdgcn_readfirstlane(uint32_t(reinterpret_cast<uintptr_t>((LDS_PTR(void))(buf + wave * 512))));
  };
  const uint32_t lds_k0 = lds_base(sK0), lds_k1 = lds_base(sK1), lds_v0 = lds_base(sV0), lds_v1 = lds_base(sV1);
  auto issue = [&](const uint16_t* base, uint16_t* stage, bool is_v, int tile, int blk) {
    const uint64_t src = reinterpret_cast<uint64_t>(base + (int64_t(blk) * BM + (tile % STEPS) * KN) * D);
    const uint32_t lds0 = stage == sK0 ? lds_k0 : stage == sK1 ? lds_k1 : stage == sV0 ? lds_v0 : lds_v1;
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int P = is_v ? PV : PK;
      const uint32_t voff = is_v ? v_off[j % PV] : k_off[j % PK];
      const uint64_t sj = src + uint64_t(j / P) * (P * RJ) * D * 2;
      const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(sj)), hi = __builtin_amdgcn_readfirstlane(uint32_t(sj >> 32));
      const uint64_t sbase = (uint64_t(hi) << 32) | lo;
      const uint32_t lds = lds0 + uint32_t(j * NW * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(sbase) : "memory", "m0");
    }
  };

  // LDS read offsets (elements), loop invariant
  const int k_sw = swz_k<CH>(n);                                    // rows 32 t + n: swizzle depends on n only
  const int v_r = (lane & 15) >> 2;                                 // row inside the 4-row group
  const int v_row = 4 * h + v_r;
  const int v_sw = swz_v<CH>(v_r);                                  // rows 16 s + 4 h + v_r (+8): same swizzle
  const int v_c = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);        // chunk inside the 32-column group
  const int v_b = (lane & 1) * 4;                                   // 8-byte half of the chunk

  // The loop works on half tiles (32 key rows).  Logits of a half tile for query tile a:
  // sx[a][i] = logit(key row 32 half + 8 (i/4) + 4 h + i%4, query row 32 a + n).
  auto k_frag = [&](const uint16_t* tK, int kk) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&tK[((2 * kk + h) ^ k_sw) * 8]));
  };
  // One product piece of O^T += V^T P^T for a half tile: piece j = (D/32) s2 + dt.  Product step s2
  // covers key rows 16 s2 + {4h..4h+3} and 16 s2 + 8 + {4h..4h+3}, which is what registers 8 s2 .. 8 s2 + 7
  // of the logit tile hold; the transposing LDS read hands each lane four consecutive key rows of one
  // value column.
  auto v_frag = [&](const uint16_t* tV, int j) {
    const int s2 = j / (D / 32), dt = j % (D / 32);
    const uint16_t* p0 = &tV[16 * s2 * D + ((4 * dt + v_c) ^ v_sw) * 8];
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(p0 + 8 * D));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto logits = [&](const uint16_t* kbuf, int half, f32x16 (&sx)[QT]) {
    const uint16_t* tK = kbuf + (32 * half + n) * D;
#pragma unroll
    for (int a = 0; a < QT; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) sx[a][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const bf16x8 f = k_frag(tK, kk);
#pragma unroll
      for (int a = 0; a < QT; ++a) sx[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[a][kk], sx[a], 0, 0, 0);
    }
  };
  // pad keys of a ragged block never count.  Only two blocks can be ragged, the last video block and the last text
  // block; their ids and real-row counts are worked out once, so that the check per half tile is two scalar compares
  // on a block id that is already at hand (measured: the 64-bit arithmetic of the general form, twice per tile, cost
  // 2 % of the kernel).
  const int real_v_last = block_real_rows(M_v - 1, BM, M_v, N_v, n_text);
  const int real_x_last = M > M_v ? block_real_rows(M - 1, BM, M_v, N_v, n_text) : BM;
  const int ragged_v = real_v_last < BM ? M_v - 1 : -1, ragged_x = real_x_last < BM ? M - 1 : -1;
  auto mask_pads = [&](int blk, int tile, int half, f32x16 (&sx)[QT]) {
    if (__builtin_expect(blk == ragged_v || blk == ragged_x, 0)) {
      asm volatile("");                               // keeps this a branch: turned into selects it would run on every half tile
      const int real = blk == ragged_v ? real_v_last : real_x_last;
      const int base = (tile % STEPS) * KN + 32 * half;
#pragma unroll
      for (int a = 0; a < QT; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (base + 8 * (i / 4) + 4 * h + (i % 4) >= real) sx[a][i] = -INFINITY;
    }
  };

  // One pipeline stage, written out in issue order.  Fragments alternate between V^T of the previous
  // half tile (products O^T += V^T P^T with its probabilities `pp`) and K of the next half tile (logit
  // chains into `sn`); every fragment feeds one matrix instruction per query tile.  In the shadow of
  // the matrix instructions the vector units run slices of the online softmax of the current half tile
  // `sx` (this lane and lane^32 hold the two halves of a query row's keys), producing `pc`.  The
  // reference maximum only moves when the row maximum outgrows it by more than 2^TAU, so the
  // accumulators are rescaled rarely; probabilities stay below 2^TAU, which is exact in the final
  // ratio.  Scheduling fences and empty asm statements keep the compiler from separating the matrix and
  // vector work again.  alpha[a] is the factor accumulator a must be multiplied by after the stage.
  auto stage = [&](auto do_pv, auto do_s, const uint16_t* vbuf, int pv_half, const u32x4 (&pp)[QT][2], const uint16_t* kbuf,
                   int s_half, f32x16 (&sn)[QT], const f32x16 (&sx)[QT], u32x4 (&pc)[QT][2], float (&alpha)[QT], bool (&moved)[QT]) {
    constexpr bool DO_PV = decltype(do_pv)::value, DO_S = decltype(do_s)::value;
    const uint16_t* tV = vbuf + (32 * pv_half + v_row) * D + v_b;
    const uint16_t* tK = kbuf + (32 * s_half + n) * D;
    bf16x8 frag[NF];
    auto load = [&](int f) {
      if (f % 2 == 0) {
        if (DO_PV) frag[f] = v_frag(tV, f / 2);
      } else if (DO_S) {
        frag[f] = k_frag(tK, f / 2);
      }
    };
    float mx_a = 0.f, mx_b = 0.f, mx_c = 0.f, mx_d = 0.f, mx = 0.f, mc = 0.f, psum = 0.f, xsum = 0.f;
    bool move = false;
    float pe[16];
    // Rounds a pair of probabilities to bf16 and adds them, as rounded, to the normaliser: numerator and
    // denominator then use exactly the same weights, so a dominant key leaves no systematic rounding bias.
    // The pair is one 32-bit register of the next product's B operand.
    auto pack = [&](int a, int i) {
      const bf16x2 pk = {(__bf16)pe[i], (__bf16)pe[i + 1]};
      psum = __builtin_amdgcn_fdot2_f32_bf16(pk, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, psum, false);
      if (XLSE) xsum += pe[i] + pe[i + 1];
      pc[a][i / 8][(i % 8) / 2] = __builtin_bit_cast(uint32_t, pk);
    };
    if (DO_S) {
#pragma unroll
      for (int a = 0; a < QT; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) sn[a][i] = 0.f;
    }
    constexpr int AHEAD = 3;                          // fragments requested ahead of their matrix instruction (2: 1 % slower;
                                                      // 4 needs two registers more than there are)
#pragma unroll
    for (int f = 0; f < AHEAD; ++f) load(f);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < STAGE_LEN; ++m) {
      if (m < SLOTS) {
        const int f = m / QT, a = m % QT;
        if (a == 0 && f + AHEAD < NF) load(f + AHEAD);
        if (f % 2 == 0) {
          if (DO_PV) {
            const int j = f / 2, s2 = j / (D / 32), dt = j % (D / 32);
            oacc[a][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[f], __builtin_bit_cast(bf16x8, pp[a][s2]), oacc[a][dt], 0, 0, 0);
          }
        } else if (DO_S) {
          sn[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[f], qf[a][f / 2], sn[a], 0, 0, 0);
        }
      }
      if (m < SLICES) {
        const int a = m / SL, ph = m % SL;
        const f32x16& x = sx[a];
        if (ph == 0) {
          mx_a = max3(x[0], x[1], x[2]);
          mx_b = max3(x[3], x[4], x[5]);
          mx_c = max3(x[6], x[7], x[8]);
          mx_d = max3(x[9], x[10], x[11]);
          psum = 0.f;
          xsum = 0.f;
        } else if (ph == 1) {
          mx_a = max3(mx_a, mx_b, mx_c);
          mx_d = max3(mx_d, x[12], x[13]);
          mx_a = max3(mx_a, x[14], x[15]);
          mx = max2(mx_a, mx_d);
          asm volatile("" : "+v"(mx));                 // keeps the slice in its slot (its result is needed only later)
        } else if (ph == 2) {
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
          mx = max2(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * c2;
          asm volatile("" : "+v"(mx));
        } else if (ph == 3) {
          move = mx - m_run[a] > TAU;                  // true on the first real half tile (m_run = M_START)
          mc = move ? mx : m_run[a];
          asm volatile("" : "+v"(mc));
        } else if (ph < 4 + ESL) {                    // the sixteen probabilities, spread evenly over ESL slices
          const int eb = (ph - 4) * 16 / ESL, ee = (ph - 3) * 16 / ESL;
#pragma unroll
          for (int i = eb; i < ee; ++i) {
            pe[i] = __builtin_amdgcn_exp2f(fmaf(x[i], c2, -mc));
            asm volatile("" : "+v"(pe[i]));
          }
          if (ph > 4) {                               // pairs completed by the previous slice: its exponentials have retired
            const int pb = (ph - 5) * 16 / ESL, pe_ = (ph - 4) * 16 / ESL;
#pragma unroll
            for (int i = pb; i < pe_; ++i)
              if (i % 2 == 1) pack(a, i - 1);
          }
        } else {
#pragma unroll
          for (int i = (ESL - 1) * 16 / ESL; i < 16; ++i)
            if (i % 2 == 1) pack(a, i - 1);
          alpha[a] = __builtin_amdgcn_exp2f(m_run[a] - mc);              // 1 unless the maximum moved
          moved[a] = __builtin_amdgcn_ballot_w64(move) != 0;
          m_run[a] = mc;
          l_run[a] = l_run[a] * alpha[a] + psum;
          if (XLSE) x_run[a] = x_run[a] * alpha[a] + xsum;
          asm volatile("" : "+v"(l_run[a]), "+v"(alpha[a]));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // accumulators *= alpha, in place (the multiply is tied to its register so that the accumulators keep
  // one home across the rarely taken branch)
  auto rescale = [&](const float (&alpha)[QT], const bool (&moved)[QT]) {
#pragma unroll
    for (int a = 0; a < QT; ++a)
      if (moved[a]) {
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float x = oacc[a][dt][i];
            asm volatile("v_mul_f32 %0, %1, %0" : "+v"(x) : "v"(alpha[a]));
            oacc[a][dt][i] = x;
          }
      }
  };
  using yes = std::true_type;
  using no = std::false_type;

  // Software pipeline over half tiles.  K(t+2) and V(t+1) are requested once per tile, right after the
  // barrier in the middle of tile t, into the buffers K(t) and V(t-1) have just left; they are first
  // read a full tile later.
  f32x16 s0[QT], s1[QT];
  u32x4 p0[QT][2], p1[QT][2];                      // probabilities as bf16 pairs: B operands of the products
  int b_cur = 0, b_nxt = 0;                        // key blocks of tiles t and t + 1: one list lookup per tile (that of tile t + 2)
  auto tile_step = [&](auto parity, auto first, auto last, int t) {
    constexpr bool ODD = decltype(parity)::value, FIRST = decltype(first)::value, LAST = decltype(last)::value;
    uint16_t* k_cur = ODD ? sK1 : sK0;             // K(t); K(t+2) goes here
    uint16_t* k_nxt = ODD ? sK0 : sK1;             // K(t+1)
    uint16_t* v_cur = ODD ? sV1 : sV0;             // V(t)
    uint16_t* v_nxt = ODD ? sV0 : sV1;             // V(t-1); V(t+1) goes here
    float alpha[QT];
    bool moved[QT];
    // first half: products of (t-1, 1), logits of (t, 1), softmax of (t, 0)
    stage(std::integral_constant<bool, !FIRST>{}, yes{}, v_nxt, 1, p1, k_cur, 1, s1, s0, p0, alpha, moved);
    rescale(alpha, moved);
    mask_pads(b_cur, t, 1, s1);
    __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): this wave's parts of K(t+1) and V(t) landed
    __syncthreads();                                 // all parts landed; every wave is past the first half of tile t
    int b_new = b_nxt;
    if (!LAST) {
      if (t + 2 < n_tiles) {
        b_new = tile_block(t + 2);
        issue(kh, k_cur, false, t + 2, b_new);
      }
      issue(vh, v_nxt, true, t + 1, b_nxt);
    }
    // second half: products of (t, 0), logits of (t+1, 0), softmax of (t, 1)
    stage(yes{}, std::integral_constant<bool, !LAST>{}, v_cur, 0, p0, k_nxt, 0, s0, s1, p1, alpha, moved);
    rescale(alpha, moved);
    if (!LAST) mask_pads(b_nxt, t + 1, 0, s0);
    b_cur = b_nxt;
    b_nxt = b_new;
  };
  if (n_tiles > 0) {
    b_cur = tile_block(0);
    b_nxt = n_tiles > 1 ? tile_block(1) : b_cur;
    issue(kh, sK0, false, 0, b_cur);
    issue(vh, sV0, true, 0, b_cur);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (n_tiles > 1) issue(kh, sK1, false, 1, b_nxt);
    logits(sK0, 0, s0);
    mask_pads(b_cur, 0, 0, s0);
    if (n_tiles == 1) {
      tile_step(no{}, yes{}, yes{}, 0);
    } else {
      tile_step(no{}, yes{}, no{}, 0);
      int t = 1;
      for (; t + 2 < n_tiles; t += 2) {              // middle tiles in pairs: buffer parities are compile-time
        tile_step(yes{}, no{}, no{}, t);
        tile_step(no{}, no{}, no{}, t + 1);
      }
      if (t + 1 < n_tiles) { tile_step(yes{}, no{}, no{}, t); ++t; }
      if (t & 1) tile_step(yes{}, no{}, yes{}, t);
      else tile_step(no{}, no{}, yes{}, t);
    }
    // drain: products of the last half tile
    const uint16_t* tV = ((n_tiles - 1) & 1 ? sV1 : sV0) + (32 + v_row) * D + v_b;
#pragma unroll
    for (int j = 0; j < 2 * (D / 32); ++j) {
      const bf16x8 f = v_frag(tV, j);
#pragma unroll
      for (int a = 0; a < QT; ++a)
        oacc[a][j % (D / 32)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, __builtin_bit_cast(bf16x8, p1[a][j / (D / 32)]), oacc[a][j % (D / 32)], 0, 0, 0);
    }
  }

  if (clock_probe && tid == 0) {
    atomicAdd(&clock_probe[0], clock64() - probe_c0);
    atomicAdd(&clock_probe[1], wall_clock64() - probe_w0);
    atomicAdd(&clock_probe[2], 1ull);
  }
  // epilogue: normalise, round to bf16, store.  Lane (n, h) holds O[row][32 dt + 8 j + 4 h + 0..3].
#pragma unroll
  for (int a = 0; a < QT; ++a) {
    const float l_tot = l_run[a] + __shfl_xor(l_run[a], 32, 64);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    uint16_t* orow = o + io_off + (io_row[a] < 0 ? 0 : io_row[a]) * D;
    if (io_row[a] >= 0) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[a][dt][4 * j + e] * inv);
          *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * j + 4 * h) = __builtin_bit_cast(u32x2, w);
        }
    }
    if (XLSE) {
      const float x_tot = x_run[a] + __shfl_xor(x_run[a], 32, 64);
      if (lse && h == 0)
        lse[int64_t(head) * N_pad + q_row0 + 32 * a] =
            x_tot > 0.f ? (m_run[a] + __builtin_amdgcn_logf(x_tot)) * 0.6931471805599453f : -INFINITY;
    }
  }
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

static unsigned long long* g_clock_probe = nullptr;   // set by dfs_attn_clock_probe (diagnostic)

int run_sparse_attn(const dfs_geom* g, const dfs_sizes& s, int dtype, const void* q, const void* k, const void* v,
                    const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale, void* o, float* lse,
                    const int32_t* row_index, hipStream_t st) {
  if (K_max < 1) return fail(DFS_ESHAPE, "dfs_sparse_attn_fwd: K_max=%d must be positive", K_max);
  if (dtype == DFS_BF16) {
    const int64_t total = int64_t(g->heads) * s.M;
    if (total > (int64_t(1) << 30)) return fail(DFS_ESHAPE, "dfs_sparse_attn_fwd: heads*M too large");
    // an eighth of a head's video blocks per XCD once that fills the XCD's 64 work-group slots (measured
    // +3..6 % on the 75 600- and 118 800-token shapes, -4 % on the 17 550-token one, which stays on mapping 1)
    const int chunk = (s.M_v + 7) / 8;
    const int mapping = chunk >= 64 ? 2 : 1;
    const int per_xcd = mapping == 2 ? (g->heads * s.M_x + 7) / 8 + g->heads * chunk : int((total + 7) / 8);
    dim3 grid(unsigned(per_xcd * 8));
#define ATTN_X(DD, BB, QQ, XX)                                                                                                  \
  attn_bf16_kernel<DD, BB, QQ, XX><<<grid, BB * 2 / QQ, 0, st>>>(static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), \
                                                                 static_cast<const uint16_t*>(v), kv_idx, kv_cnt, K_max,          \
                                                                 static_cast<uint16_t*>(o), lse, row_index, s.N, s.N_pad, s.N_v,  \
                                                                 g->n_text, s.M_v, s.M, int(total), per_xcd, mapping, scale, g_clock_probe)
#define ATTN(DD, BB, QQ) do { if (lse) ATTN_X(DD, BB, QQ, true); else ATTN_X(DD, BB, QQ, false); } while (0)
    if (g->d == 64) { if (g->B == 64) ATTN(64, 64, 1); else ATTN(64, 128, 1); }
    else            { if (g->B == 64) ATTN(128, 64, 1); else ATTN(128, 128, 1); }
#undef ATTN
#undef ATTN_X
  } else {
    if (row_index) return fail(DFS_EDTYPE, "dfs_sparse_attn_fwd: reading Q / writing O through the permutation needs bf16 tensors");
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

extern "C" int dfs_attn_clock_probe(uint64_t* counters) {
  if (misaligned(8, {counters})) return fail(DFS_EINVAL, "dfs_attn_clock_probe: counters must be 8-byte aligned");
  g_clock_probe = reinterpret_cast<unsigned long long*>(counters);
  return DFS_OK;
}

extern "C" int dfs_sparse_attn_fwd(const dfs_geom* g, int dtype, const void* q_perm, const void* k_perm, const void* v_perm,
                                   const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale, void* o_perm,
                                   float* lse, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_F32 && dtype != DFS_BF16) return fail(DFS_EDTYPE, "dtype %d is not DFS_F32 or DFS_BF16", dtype);
  if (!q_perm || !k_perm || !v_perm || !kv_idx || !kv_cnt || !o_perm) return fail(DFS_EINVAL, "dfs_sparse_attn_fwd: NULL argument");
  if (misaligned(16, {q_perm, k_perm, v_perm, o_perm}) || misaligned(4, {kv_idx, kv_cnt, lse}))
    return fail(DFS_EINVAL, "dfs_sparse_attn_fwd: tensors must be 16-byte aligned, index and fp32 arrays 4-byte aligned");
  if (!(scale > 0.f)) return fail(DFS_EINVAL, "dfs_sparse_attn_fwd: scale must be positive");
  return run_sparse_attn(g, s, dtype, q_perm, k_perm, v_perm, kv_idx, kv_cnt, K_max, scale, o_perm, lse, nullptr, as_stream(stream));
}

extern "C" int dfs_sparse_attn_fwd_src(const dfs_geom* g, int dtype, const void* q, const int32_t* perm_pad, const void* k_perm,
                                       const void* v_perm, const int32_t* kv_idx, const int32_t* kv_cnt, int32_t K_max, float scale,
                                       void* o, float* lse, void* stream) {
  dfs_sizes s;
  int rc = check_geom(g, &s);
  if (rc) return rc;
  if (dtype != DFS_BF16) return fail(DFS_EDTYPE, "dfs_sparse_attn_fwd_src: bf16 tensors only");
  if (!q || !perm_pad || !k_perm || !v_perm || !kv_idx || !kv_cnt || !o) return fail(DFS_EINVAL, "dfs_sparse_attn_fwd_src: NULL argument");
  if (misaligned(16, {q, k_perm, v_perm, o}) || misaligned(4, {perm_pad, kv_idx, kv_cnt, lse}))
    return fail(DFS_EINVAL, "dfs_sparse_attn_fwd_src: tensors must be 16-byte aligned, index and fp32 arrays 4-byte aligned");
  if (!(scale > 0.f)) return fail(DFS_EINVAL, "dfs_sparse_attn_fwd_src: scale must be positive");
  return run_sparse_attn(g, s, dtype, q, k_perm, v_perm, kv_idx, kv_cnt, K_max, scale, o, lse, perm_pad, as_stream(stream));
}
