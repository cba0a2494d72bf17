// Causal window attention over the paged KV cache (grouped-query), bf16 MFMA
// with fp32 online softmax.
//
// Reduction schedule of one query row at absolute position p (it depends on p
// and on nothing else - not on the window, the row's index in it, the batch, or
// the context lengths of other sequences).  Keys are cut at absolute positions:
//   step   = 64 keys   [64 j, 64 j + 64)
//   chunk  = 256 keys  = 4 steps
//   super  = 2048 keys = 8 chunks
// * A chunk partial (m, l, acc) starts at (-inf, 0, 0) and is advanced by one
//   online-softmax step per 64 keys in ascending order; a step computes its
//   scores with head_dim/32 MFMA k-steps per 16-key block, takes max and sum
//   over its 64 keys in a fixed tree, rescales, and adds P V with two MFMA
//   k-steps of 32 keys.
// * The chunk partials of a super are folded left to right (fold() below), giving
//   the super partial; the super partials are folded left to right, giving the row.
// Keys beyond p contribute exact zeros (masked before the exponential); a step or
// a chunk in which every key of a row is masked leaves that row's state bit for
// bit unchanged, so rows of different positions can share a workgroup.
//
// Work distribution (free to change, does not touch the bits): a workgroup owns one unit of the keys
// of a (sequence, kv head) for 8 blocks of 16 query rows (attention_stream_kernel, 8 waves) or up to 4
// (attention_kernel, 4 waves); query rows are ordered r = q_head_in_group * window + i.  A unit is
//   a chunk          - few sequences: most parallelism; chunk partials are written and the merge
//                      kernel does all folds;
//   a super          - more sequences: chunks are folded in registers, 8 times fewer partials;
//   a whole sequence - many sequences whose lengths deal out evenly (the plan kernel decides from the
//                      lengths): supers are folded in registers too and the workgroup writes the
//                      output rows itself, as it does whenever every context fits one super.
// K and V tiles go from global memory straight into a ring of LDS entries of 64 keys, three entries in
// flight, already in MFMA operand order (see the KV tile layouts in llm42.h), so nothing is transposed.
#include <algorithm>
#include <type_traits>

#include "llm42_dev.h"

namespace {

constexpr int STEP = 64, CHUNK = 256, SUPER_KEYS = 2048;
constexpr float kLazy = 8.0f;   // log2 units, see softmax_step

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;

// state <- state (+) part, the only way two partials are ever combined:
//   mn = max(M, m2), a = exp2(M - mn), b = exp2(m2 - mn), L = fma(l2, b, L * a), A = fma(a2, b, A * a).
// One of a, b is exactly 1; where a is 1 for every lane of the wave (the running maximum stands,
// the usual case) the multiplication by it is left out, which cannot change a bit.
template <int NV>
__device__ inline void fold(float& M, float& L, f32x4 (&A)[NV], float m2, float l2, const f32x4 (&a2)[NV]) {
  const float mn = fmaxf(M, m2);
  const float mu = mn == -INFINITY ? 0.f : mn;
  const float a = __builtin_amdgcn_exp2f(M - mu), b = __builtin_amdgcn_exp2f(m2 - mu);
  if (__builtin_amdgcn_ballot_w64(a != 1.0f) != 0) {
    L *= a;
#pragma unroll
    for (int i = 0; i < NV; ++i) A[i] *= a;
  }
  L = __builtin_fmaf(l2, b, L);
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int c = 0; c < 4; ++c) A[i][c] = __builtin_fmaf(a2[i][c], b, A[i][c]);
  M = mn;
}

// Copy one KV tile (TL KiB) from global memory to LDS without passing through registers: one
// instruction moves 1 KiB, lane i's 16 bytes landing at LDS byte address `dst` + 16 i (M0 holds the
// wave-uniform destination).  `src` already includes this lane's 16-byte offset.  Written as
// assembly on purpose: with the compiler's own form of this load every later LDS read waits for
// all earlier ones, which un-pipelines the operand reads of the steps.  The compiler therefore
// does not count these loads; fetch_landed() is the only wait that covers them.  Nothing else in
// this kernel uses M0.  STREAM marks the load non-temporal: K and V tiles are read once per (sequence,
// kv head) and launch, and the hint takes the fetch stream alone (no arithmetic) from 5.1 to 5.7 TB/s.
template <int TL, bool STREAM = false>
__device__ __forceinline__ void tile_to_lds(uint32_t dst, const uint4* src) {
#pragma unroll
  for (int i = 0; i < TL; ++i)
    if constexpr (STREAM)
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                   :
                   : "v"(src + i * 64), "s"(dst + i * 1024)
                   : "memory", "m0");
    else
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                   :
                   : "v"(src + i * 64), "s"(dst + i * 1024)
                   : "memory", "m0");
}
// At most N of the fetches this wave has issued are still on their way (they complete in order;
// the barrier that follows covers the other waves').
template <int N>
__device__ __forceinline__ void fetch_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
// Every fetch this wave has issued is in LDS.
// (Both forms of the wait: the first tells the compiler that its own loads are complete as well.)
__device__ __forceinline__ void fetch_landed() {
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Butterflies over the four 16-lane rows of a wave (lane ^ 16, then lane ^ 32) without a trip
// through LDS: a swap leaves the two partners of every lane in the two results, and max / + are
// commutative, so each lane gets the same bits as from the shuffle form of the butterfly.
__device__ __forceinline__ float rows_max(float x) {
  u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float rows_sum(float x) {
  u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(r.x) + __uint_as_float(r.y);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);
}

// The output of query row r (of sequence s, kv head kvh): acc / l in bf16, into the tile layout of the
// O-projection's activation operand - exactly what the merge pass computes from a row's folded partials.
// The lane holds features d * 16 + g * 4 .. + 3 of the row; the lanes g and g ^ 1 of a row trade halves so that each
// writes 8 consecutive features of every second block d (16 bytes per lane and store, half as many stores).
// Called by all four lanes of a row or by none.
template <int HD>
__device__ __forceinline__ void store_output(uint16_t* __restrict__ out, int d_attn, int s, int kvh, int group, int window,
                                             int r, int g, const f32x4 (&acc)[HD / 16], float l) {
  const int i = r % window, hq = kvh * group + r / window;
  const bool odd = g & 1;
#pragma unroll
  for (int d = 0; d < HD / 16; d += 2) {
    const uint32_t a0 = pack2_bf16(acc[d][0] / l, acc[d][1] / l), a1 = pack2_bf16(acc[d][2] / l, acc[d][3] / l);
    const uint32_t b0 = pack2_bf16(acc[d + 1][0] / l, acc[d + 1][1] / l), b1 = pack2_bf16(acc[d + 1][2] / l, acc[d + 1][3] / l);
    // even g keeps block d and takes its neighbour's four features of it; odd g keeps block d + 1
    const uint32_t t0 = __shfl_xor(odd ? a0 : b0, 16), t1 = __shfl_xor(odd ? a1 : b1, 16);
    const u32x4 o = odd ? (u32x4){t0, t1, b0, b1} : (u32x4){a0, a1, t0, t1};
    *(u32x4*)(out + pk_off(s * window + i, hq * HD + (d + (odd ? 1 : 0)) * 16 + (g & 2) * 4, d_attn)) = o;
  }
}

// One online-softmax step over the 64 keys [k0, k0 + 64): `lk` / `lv` are the step's four K and
// four V tiles in LDS.  MASKED = false is the same arithmetic with the comparisons that cannot
// fail left out: every key of the step is at or below every position of this wave's rows (and
// hence below k_hi).  The operand reads are issued one ring ahead of the MFMAs that consume them
// and the order is pinned, so that an LDS round trip is never waited for in full.
template <int HD, int CB, bool MASKED>
__device__ __forceinline__ void softmax_step(const uint4* lk, const uint16_t* lv, int k0, int k_hi, int lane,
                                             float scale_log2, const bf16x8 (&qf)[CB][HD / 32], const int (&qpos)[CB],
                                             float (&m)[CB], float (&l)[CB], f32x4 (&acc)[CB][HD / 16], const bool first) {
  constexpr int DK = HD / 32, DB = HD / 16, TV4 = HD * 2;
  const int col = lane & 15, g = lane >> 4;
  constexpr int RV = 4;                                     // V operands in flight
  bf16x8 kb[DK];                                            // K operands in flight, one per head-dim k-step
  u32x4 vb[RV];
  auto load_k = [&](int b, int d) { kb[d] = ((const bf16x8*)lk)[b * TV4 + d * 64 + lane]; };
  auto load_v = [&](int idx) {                              // idx = key pair kk * DB + feature block d
    const uint16_t* vt0 = lv + (size_t)(2 * (idx / DB)) * TV4 * 8 + (((idx % DB) * 4 + g) * 16 + col) * 4;
    const u32x2 lo = *(const u32x2*)vt0, hi = *(const u32x2*)(vt0 + TV4 * 8);
    vb[idx % RV] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
  };
  // ---- raw scores of 4 blocks of 16 keys: S^T[key][query] ---------------------------------
  f32x4 sc[CB][4];
#pragma unroll
  for (int d = 0; d < DK; ++d) load_k(0, d);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int b = 0; b < 4; ++b) {
#pragma unroll
    for (int d = 0; d < DK; ++d) {
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
        sc[cb][b] = mfma16(kb[d], qf[cb][d], d == 0 ? (f32x4){0.f, 0.f, 0.f, 0.f} : sc[cb][b]);
      if (b + 1 < 4) load_k(b + 1, d);
      else if (d < RV) load_v(d);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int i = DK; i < RV; ++i) load_v(i);
  // ---- mask, online softmax state (m in units of scaled scores), P in bf16 -----------------
  u32x4 pf[CB][2];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (MASKED) {
      // a select, not arithmetic: scores of keys past k_hi come from stale tiles and may be anything
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (k0 + b * 16 + g * 4 + e > qpos[cb]) sc[cb][b][e] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(sc[cb][0][0], sc[cb][0][1]), sc[cb][0][2]);
    mx = fmaxf(fmaxf(mx, sc[cb][0][3]), sc[cb][1][0]);
    mx = fmaxf(fmaxf(mx, sc[cb][1][1]), sc[cb][1][2]);
    mx = fmaxf(fmaxf(mx, sc[cb][1][3]), sc[cb][2][0]);
    mx = fmaxf(fmaxf(mx, sc[cb][2][1]), sc[cb][2][2]);
    mx = fmaxf(fmaxf(mx, sc[cb][2][3]), sc[cb][3][0]);
    mx = fmaxf(fmaxf(mx, sc[cb][3][1]), sc[cb][3][2]);
    mx = rows_max(fmaxf(mx, sc[cb][3][3]));
    // scaling by a positive constant is monotonic: max(scaled) == scaled(max), bit for bit
    const float m_step = mx * scale_log2;
    // The partial's reference exponent m moves up to this step's maximum only when that exceeds it by more than
    // kLazy (then p = exp2(score - m) stays at or below 2^kLazy); otherwise it stands and alpha is exactly 1.
    // (An empty partial has m = -inf: +inf > kLazy takes the step's maximum; -inf - -inf is NaN and keeps -inf.)
    const float m_new = (m_step - m[cb] > kLazy) ? m_step : m[cb];
    const float m_use = (MASKED && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m[cb] - m_use);
    float rs = 0.f;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        sc[cb][b][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[cb][b][e], scale_log2, -m_use));
      rs += ((sc[cb][b][0] + sc[cb][b][1]) + sc[cb][b][2]) + sc[cb][b][3];
    }
    rs = rows_sum(rs);
    // Rescaling by alpha is skipped where it cannot change a bit: in the first step of a partial (l and acc are
    // zero, and zero times alpha is zero) and where alpha is exactly 1 for every row of the wave.
    if (!first && __builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
      l[cb] *= alpha;
#pragma unroll
      for (int d = 0; d < DB; ++d) acc[cb][d] *= alpha;
    }
    l[cb] += rs;
    m[cb] = m_new;
    // k-slot e of lane group g is key g*4+e of the first block of a pair (e < 4) or of the
    // second (e >= 4); V uses the same assignment
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      pf[cb][kk][0] = pack2_bf16(sc[cb][2 * kk][0], sc[cb][2 * kk][1]);
      pf[cb][kk][1] = pack2_bf16(sc[cb][2 * kk][2], sc[cb][2 * kk][3]);
      pf[cb][kk][2] = pack2_bf16(sc[cb][2 * kk + 1][0], sc[cb][2 * kk + 1][1]);
      pf[cb][kk][3] = pack2_bf16(sc[cb][2 * kk + 1][2], sc[cb][2 * kk + 1][3]);
    }
  }
  // ---- acc^T[feature][query] += V^T P^T, 32 keys per MFMA ------------------------------
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int idx = 0; idx < 2 * DB; ++idx) {
    const int kk = idx / DB, d = idx % DB;
    if (MASKED) {
      // slots at or beyond k_hi hold stale, never-written or foreign data: force them to zero
      // so that 0 * garbage cannot produce a NaN
      const int kp0 = k0 + kk * 32 + g * 4, kp1 = kp0 + 16;
      if (kp1 + 3 >= k_hi) {
        u32x4& v = vb[idx % RV];
        if (kp0 + 0 >= k_hi) v[0] &= 0xFFFF0000u;
        if (kp0 + 1 >= k_hi) v[0] &= 0x0000FFFFu;
        if (kp0 + 2 >= k_hi) v[1] &= 0xFFFF0000u;
        if (kp0 + 3 >= k_hi) v[1] &= 0x0000FFFFu;
        if (kp1 + 0 >= k_hi) v[2] &= 0xFFFF0000u;
        if (kp1 + 1 >= k_hi) v[2] &= 0x0000FFFFu;
        if (kp1 + 2 >= k_hi) v[3] &= 0xFFFF0000u;
        if (kp1 + 3 >= k_hi) v[3] &= 0x0000FFFFu;
      }
    }
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      acc[cb][d] = mfma16(__builtin_bit_cast(bf16x8, vb[idx % RV]), __builtin_bit_cast(bf16x8, pf[cb][kk]),
                          acc[cb][d]);
    if (idx + RV < 2 * DB) load_v(idx + RV);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int HD, int CB, int NW, bool SUPER>
__global__ __launch_bounds__(NW * 64) void attention_kernel(
    const uint16_t* __restrict__ q, const uint4* __restrict__ k_plane, const uint4* __restrict__ v_plane,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_len, const int32_t* __restrict__ seq_n,
    const int4* __restrict__ items, const int32_t* __restrict__ item_count, int32_t* __restrict__ queue,
    int n_kv_heads, int group, int window, int r_pad, int y_blocks, int max_blocks_per_seq, int n_units,
    float scale_log2, float* __restrict__ part_acc, float* __restrict__ part_ml, uint16_t* __restrict__ attn_out,
    int d_attn) {
  constexpr int DK = HD / 32;        // MFMA k-steps over the head dimension (scores)
  constexpr int DB = HD / 16;        // 16-feature blocks of the output
  constexpr int TV4 = HD * 2;        // uint4 per KV tile (16 tokens x HD bf16)
  constexpr int TL = TV4 / 64;       // uint4 per lane per tile
  constexpr int UNIT = SUPER ? SUPER_KEYS : CHUNK;
  constexpr int NBUF = 4, AHEAD = 3;    // ring of step buffers; steps in flight ahead of the one computed
  constexpr int FI = 8 * TL / NW;       // fetch instructions per wave per step (4 K and 4 V tiles in all)
  static_assert(NW == 4 || NW == 8, "a step's tiles are split over 4 or 8 waves");
  static_assert(TL % (NW / 4) == 0, "half a tile per wave needs an even number of pieces");
  __shared__ uint4 lds_k[NBUF][4 * TV4];   // per step: 4 K tiles
  __shared__ uint4 lds_v[NBUF][4 * TV4];   // and 4 V tiles
  __shared__ int wg_max[NW];
  __shared__ int next_work;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(lds_ptr)&lds_k[0][0];
  const uint32_t lds_v_addr = (uint32_t)(uintptr_t)(lds_ptr)&lds_v[0][0];

  // One work item: unit `unit` of the keys of sequence `s`, kv head `kvh`, for the `yb`-th group of
  // NW * CB blocks of 16 query rows.  (A return leaves the item; every condition is workgroup-uniform.)
  auto run_item = [&](const int unit, const int yb, const int s, const int kvh) {
  const int k_lo = unit * UNIT;
  const int32_t* bt = block_table + (size_t)s * max_blocks_per_seq;
  // Requested before anything is known about the sequence, so that the three latencies (lengths,
  // block ids, query operands) overlap: the unit's block-table entries (clamped to the table, not
  // yet to the sequence) and the query operands of this wave's row blocks.
  const int first_blk = k_lo >> 4;
  const int raw0 = bt[min(first_blk + lane, max_blocks_per_seq - 1)];
  const int raw1 = SUPER ? bt[min(first_blk + 64 + lane, max_blocks_per_seq - 1)] : 0;
  bf16x8 qf[CB][DK];
  int row[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    row[cb] = ((yb * NW + wave) * CB + cb) * 16 + col;
    // row blocks past r_pad (grid padding) read the last real block instead; their rows are dead anyway
    const int rb = min(row[cb] >> 4, r_pad / 16 - 1);
    const uint16_t* qb = q + ((size_t)s * n_kv_heads + kvh) * r_pad * HD + (size_t)rb * DK * 512;
#pragma unroll
    for (int d = 0; d < DK; ++d) qf[cb][d] = *(const bf16x8*)(qb + d * 512 + lane * 8);
  }
  const int L = seq_len[s], n = seq_n[s];
  if (L < 0) return;                                         // whole workgroup

  int qpos[CB];
  int wmax = -1, wmin = 0x7FFFFFFF;   // highest and lowest position among this wave's rows (dead rows: -1)
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int i = row[cb] % window;
    qpos[cb] = (row[cb] < group * window && i < n) ? L + i : -1;
    wmax = max(wmax, qpos[cb]);
    wmin = min(wmin, qpos[cb]);
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    wmax = max(wmax, __shfl_xor(wmax, off));
    wmin = min(wmin, __shfl_xor(wmin, off));
  }
  wmin = __builtin_amdgcn_readfirstlane(wmin);
  if (lane == 0) wg_max[wave] = wmax;
  __syncthreads();
  int gmax = wg_max[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) gmax = max(gmax, wg_max[w]);
  if (gmax < k_lo) return;                                   // whole workgroup: nobody looks into this unit
  const int k_hi = min(gmax + 1, k_lo + UNIT);               // exclusive; <= L + n
  const int n_steps = (k_hi - k_lo + STEP - 1) / STEP;
  const int last_blk = (k_hi - 1) >> 4;
  // table entries past the last needed block may hold anything: replace them by the last needed
  // block's id (its data is fetched in their place, and every key in those positions is masked)
  const int last_id = __shfl((last_blk - first_blk) < 64 ? raw0 : raw1, (last_blk - first_blk) & 63);
  const int ids0 = first_blk + lane <= last_blk ? raw0 : last_id;
  const int ids1 = first_blk + 64 + lane <= last_blk ? raw1 : last_id;

  // each wave fetches one (4 waves) or half (8 waves) of the four blocks of a step, its K and its V
  // tile, straight from global memory into LDS
  auto fetch = [&](int j) {
    constexpr int SPLIT = NW / 4, PIECES = TL / SPLIT;       // waves per block; 1 KiB pieces per wave and tile
    const int blk = wave / SPLIT, part = wave % SPLIT;
    const int bj = j * 4 + blk;                              // block index inside the unit (wave-uniform)
    const int id = bj < 64 ? __builtin_amdgcn_readlane(ids0, bj & 63) : __builtin_amdgcn_readlane(ids1, bj & 63);
    const uint32_t off = (uint32_t)(((j & (NBUF - 1)) * 4 + blk) * TV4 + part * PIECES * 64) * 16;
    const size_t src = ((size_t)id * n_kv_heads + kvh) * TV4 + part * PIECES * 64 + lane;
    tile_to_lds<PIECES, true>(lds_k_addr + off, k_plane + src);
    tile_to_lds<PIECES, true>(lds_v_addr + off, v_plane + src);
  };

  float m[CB], l[CB];
  f32x4 acc[CB][DB];
  float sm[CB], sl[CB];                                      // super mode: running fold of finished chunks
  f32x4 sacc[CB][DB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    m[cb] = -INFINITY;
    l[cb] = 0.f;
    sm[cb] = -INFINITY;
    sl[cb] = 0.f;
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      acc[cb][d] = (f32x4){0.f, 0.f, 0.f, 0.f};
      sacc[cb][d] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
  }

  // Steps j+1 .. j+AHEAD are in flight while step j is computed.  A buffer is refilled only after the
  // barrier that ends the step which read it; the wait before that barrier leaves the younger
  // fetches in flight (loads complete in order).
#pragma unroll
  for (int j = 0; j < AHEAD; ++j)
    if (j < n_steps) fetch(j);
  fetch_landed();
  __syncthreads();
  for (int j = 0; j < n_steps; ++j) {
    if (j + AHEAD < n_steps) fetch(j + AHEAD);                // into the buffer of step j - 1
    {
      const int k0 = k_lo + j * STEP;
      const uint4* sk = &lds_k[j & (NBUF - 1)][0];
      const uint16_t* sv = (const uint16_t*)&lds_v[j & (NBUF - 1)][0];
      const bool first = SUPER ? (j & 3) == 0 : j == 0;        // the chunk partial is empty
      if (k0 + STEP - 1 <= wmin)                               // wave-uniform
        softmax_step<HD, CB, false>(sk, sv, k0, k_hi, lane, scale_log2, qf, qpos, m, l, acc, first);
      else
        softmax_step<HD, CB, true>(sk, sv, k0, k_hi, lane, scale_log2, qf, qpos, m, l, acc, first);
    }
    if (SUPER && ((j & 3) == 3 || j + 1 == n_steps)) {
      // a chunk is complete: fold it into the running super partial and start the next one afresh
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        if (j < 4) {
          sm[cb] = m[cb];
          sl[cb] = l[cb];
#pragma unroll
          for (int d = 0; d < DB; ++d) sacc[cb][d] = acc[cb][d];
        } else {
          fold<DB>(sm[cb], sl[cb], sacc[cb], m[cb], l[cb], acc[cb]);
        }
        m[cb] = -INFINITY;
        l[cb] = 0.f;
#pragma unroll
        for (int d = 0; d < DB; ++d) acc[cb][d] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    }
    // step j + 1 has landed once at most the fetches issued after it are outstanding
    const int younger = min(j + AHEAD, n_steps - 1) - (j + 1);
    if (younger >= 2) fetch_wait<2 * FI>();
    else if (younger == 1) fetch_wait<FI>();
    else fetch_wait<0>();
    __syncthreads();
  }

  // ---- partial of this unit for every row that reaches into it ---------------------------------
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (qpos[cb] < k_lo) continue;
    if (SUPER && attn_out) {   // (one unit per sequence: no partial, no merge pass)
      store_output<HD>(attn_out, d_attn, s, kvh, group, window, row[cb], g, sacc[cb], sl[cb]);
      continue;
    }
    const size_t prow = (((size_t)s * n_kv_heads + kvh) * n_units + unit) * r_pad + row[cb];
    float* pa = part_acc + prow * HD;
#pragma unroll
    for (int d = 0; d < DB; ++d) *(f32x4*)(pa + d * 16 + g * 4) = SUPER ? sacc[cb][d] : acc[cb][d];
    if (g == 0) *(float2*)(part_ml + prow * 2) = SUPER ? make_float2(sm[cb], sl[cb]) : make_float2(m[cb], l[cb]);
  }
  };  // run_item

  // Work distribution: the workgroups of the (CU-sized) grid take one item each to begin with and
  // pull further ones from a queue.  The list of (sequence, unit) pairs that hold keys is built once
  // per call (attention_plan_kernel), so no workgroup is spent on a unit past a sequence's end, and
  // the order in which workgroups finish does not matter: every item writes its own partial.
  const int per_item = n_kv_heads * y_blocks;
  const int total = *item_count * per_item;
  for (int t = blockIdx.x; t < total;) {
    const int it = t / per_item, rem = t - it * per_item;
    const int4 su = items[it];
    run_item(su.y, rem % y_blocks, su.x, rem / y_blocks);
    __syncthreads();                                       // every wave is done with the ring
    if (threadIdx.x == 0) next_work = (int)gridDim.x + atomicAdd(queue, 1);
    __syncthreads();
    t = next_work;
  }
}

// The same computation for 8 or more blocks of query rows per (sequence, kv head), as one stream per
// CU.  A workgroup of 8 waves (one block of 16 query rows each) walks its share of the work items
// (item t of round r goes to workgroup t mod G, rounds alternating direction, items sorted longest
// first: an even split without a queue).  Everything it needs from global memory arrives through one
// ring of LDS entries that never stops at an item boundary: per item first an entry with the eight
// row blocks' query operands, then one entry (4 K tiles + 4 V tiles) per 64-key step, AHEAD entries
// in flight.  A fetch cursor and a compute cursor walk the same item list independently; all item
// data they need is wave-uniform and comes through scalar loads, so nothing but the ring's own
// fetches is ever counted by vmcnt between the first and the last entry.  Past the last item the
// fetch cursor issues dummy fetches into slots nothing reads, which keeps the wait count constant.
// FOLD = false (measurement only): no chunk partials inside a super, one straight accumulation.
// SEQ: an item is a whole sequence (all of its supers); the supers' partials are folded in registers, in the order
// of the merge pass, and the kernel writes the output rows itself.  The query operands then stay in LDS instead of
// registers (the third accumulator level needs theirs).
template <int HD, bool SUPER, bool FOLD, bool SEQ = false>
__global__ __launch_bounds__(512) void attention_stream_kernel(
    const uint16_t* __restrict__ q, const uint4* __restrict__ k_plane, const uint4* __restrict__ v_plane,
    const int32_t* __restrict__ block_table, const int4* __restrict__ items, const int32_t* __restrict__ item_count,
    int n_kv_heads, int group, int window, int r_pad, int y_blocks, int max_blocks_per_seq, int n_units,
    float scale_log2, float* __restrict__ part_acc, float* __restrict__ part_ml, uint16_t* __restrict__ attn_out,
    int d_attn, const int32_t* __restrict__ seq_mode) {
  if ((*seq_mode != 0) != SEQ) return;   // the plan chose the other kind of item for this call (workgroup-uniform)
  constexpr int NW = 8, CB = 1;
  constexpr int DK = HD / 32, DB = HD / 16, TV4 = HD * 2, TL = TV4 / 64;
  constexpr int UNIT = SUPER ? SUPER_KEYS : CHUNK;
  constexpr int NBUF = 4, AHEAD = 3;
  constexpr int FI = TL;                // fetch instructions per wave per entry
  static_assert(TL % 2 == 0, "half a tile per wave");
  static_assert(!SEQ || (SUPER && FOLD), "whole sequences are folded like supers");
  __shared__ uint4 ring[NBUF][8 * TV4];
  __shared__ uint4 q_keep[SEQ ? 8 * TV4 : 1];   // SEQ: every wave's block of query operands for the current item

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const uint32_t ring_addr = (uint32_t)(uintptr_t)(lds_ptr)&ring[0][0];
  const int G = gridDim.x, w = blockIdx.x;
  const int per_item = n_kv_heads * y_blocks;
  const int total = *item_count * per_item;

  // the ord-th piece of work of this workgroup (wave-uniform; scalar loads)
  struct Work {
    bool valid;
    int s, kvh, yb, unit, L, n, k_lo, k_hi, n_steps;
  };
  auto work_of = [&](int ord) {
    Work x;
    const int t = ord * G + ((ord & 1) ? G - 1 - w : w);
    x.valid = t < total;
    const int tt = x.valid ? t : 0;
    const int it = tt / per_item, rem = tt - it * per_item;
    // (past the end: a harmless stand-in, so that the dummy fetches read valid memory)
    const int4 su = x.valid ? items[it] : make_int4(0, 0, 0, 1);
    x.s = su.x, x.unit = su.y, x.L = su.z, x.n = su.w;
    x.kvh = rem / y_blocks, x.yb = rem % y_blocks;
    x.k_lo = SEQ ? 0 : x.unit * UNIT;
    x.k_hi = SEQ ? x.L + x.n : min(x.L + x.n, x.k_lo + UNIT);
    x.n_steps = (x.k_hi - x.k_lo + STEP - 1) / STEP;
    return x;
  };

  // ---- fetch cursor ----------------------------------------------------------------------------
  int f_ord = 0, f_entry = 0;           // entry 0 = query operands, entry e > 0 = step e - 1
  Work f = work_of(0);
  int f_id = 0;                         // block id this wave needs for the entry at the cursor (steps only)
  const int blk = wave >> 1, part = wave & 1;
  auto id_for = [&](const Work& x, int e) {   // physical block of this wave's 16 keys of step e - 1
    const int b = min((x.k_lo >> 4) + (e - 1) * 4 + blk, (x.k_hi - 1) >> 4);   // never past the last block in use
    return block_table[(size_t)x.s * max_blocks_per_seq + b];
  };
  auto fetch_next = [&](int gidx) {
    const uint32_t slot = ring_addr + (uint32_t)((gidx & (NBUF - 1)) * 8 * TV4) * 16;
    if (!f.valid || f_entry == 0) {
      // this wave's block of 16 query rows (row blocks past r_pad read the last real one; past the
      // last item: the same fetch once more, into a slot nothing reads)
      const int rb = min(f.yb * NW + wave, r_pad / 16 - 1);
      const uint4* src = (const uint4*)(q + ((size_t)f.s * n_kv_heads + f.kvh) * r_pad * HD + (size_t)rb * DK * 512);
      tile_to_lds<TL>(slot + (uint32_t)(wave * TV4) * 16, src + lane);
    } else {
      const size_t src = ((size_t)f_id * n_kv_heads + f.kvh) * TV4 + part * (TL / 2) * 64 + lane;
      const uint32_t off = (uint32_t)(blk * TV4 + part * (TL / 2) * 64) * 16;
      tile_to_lds<TL / 2, true>(slot + off, k_plane + src);
      tile_to_lds<TL / 2, true>(slot + (uint32_t)(4 * TV4) * 16 + off, v_plane + src);
    }
    if (f.valid) {
      if (++f_entry > f.n_steps) {
        f = work_of(++f_ord);
        f_entry = 0;
      } else {
        f_id = id_for(f, f_entry);      // requested one entry ahead of its use
      }
    }
  };

  // ---- compute cursor ---------------------------------------------------------------------------
#pragma unroll
  for (int e = 0; e < AHEAD; ++e) fetch_next(e);
  fetch_wait<(AHEAD - 1) * FI>();       // entry 0 has landed
  __syncthreads();
  int gidx = 0;                         // ring entry being consumed
  auto entry_done = [&]() {
    fetch_wait<(AHEAD - 1) * FI>();     // the next entry has landed: only the fetches issued after it may be outstanding
    __syncthreads();                    // ... for every wave, and every wave is done with this entry's slot
    ++gidx;
  };
  Work c = work_of(0);
  for (int ord = 0; c.valid; ++ord) {
    const Work c_next = work_of(ord + 1);   // requested now, needed when this item is done
    // -- entry 0: query operands; per-lane row data
    fetch_next(gidx + AHEAD);
    bf16x8 qf[CB][DK];
#pragma unroll
    for (int d = 0; d < DK; ++d) qf[0][d] = ((const bf16x8*)ring[gidx & (NBUF - 1)])[wave * TV4 + d * 64 + lane];
    if (SEQ) {   // (each wave keeps and re-reads its own block only: no barrier needed for it)
#pragma unroll
      for (int d = 0; d < DK; ++d) ((bf16x8*)q_keep)[wave * TV4 + d * 64 + lane] = qf[0][d];
    }
    int row[CB], qpos[CB];
    row[0] = (c.yb * NW + wave) * 16 + col;
    {
      const int i = row[0] % window;
      qpos[0] = (row[0] < group * window && i < c.n) ? c.L + i : -1;
    }
    int wmin = qpos[0];               // lowest position among this wave's rows (dead rows: -1)
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) wmin = min(wmin, __shfl_xor(wmin, off));
    wmin = __builtin_amdgcn_readfirstlane(wmin);
    float m[CB] = {-INFINITY}, l[CB] = {0.f}, sm[CB] = {-INFINITY}, sl[CB] = {0.f};
    f32x4 acc[CB][DB], sacc[CB][DB];
    float tm = -INFINITY, tl = 0.f;   // SEQ: running fold of finished supers
    f32x4 tacc[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      acc[0][d] = (f32x4){0.f, 0.f, 0.f, 0.f};
      sacc[0][d] = (f32x4){0.f, 0.f, 0.f, 0.f};
      tacc[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    entry_done();
    // -- one entry per step
    for (int j = 0; j < c.n_steps; ++j) {
      fetch_next(gidx + AHEAD);
      const int k0 = c.k_lo + j * STEP;
      const uint4* sk = &ring[gidx & (NBUF - 1)][0];
      const uint16_t* sv = (const uint16_t*)&ring[gidx & (NBUF - 1)][4 * TV4];
      if (SEQ) {
#pragma unroll
        for (int d = 0; d < DK; ++d) qf[0][d] = ((const bf16x8*)q_keep)[wave * TV4 + d * 64 + lane];
      }
      const bool first = SUPER && FOLD ? (j & 3) == 0 : j == 0;   // the chunk partial is empty
      if (k0 + STEP - 1 <= wmin)                               // wave-uniform
        softmax_step<HD, CB, false>(sk, sv, k0, c.k_hi, lane, scale_log2, qf, qpos, m, l, acc, first);
      else
        softmax_step<HD, CB, true>(sk, sv, k0, c.k_hi, lane, scale_log2, qf, qpos, m, l, acc, first);
      if (SUPER && FOLD && ((j & 3) == 3 || j + 1 == c.n_steps)) {
        // a chunk is complete: fold it into the running super partial and start the next one afresh
        if ((SEQ ? (j & 31) : j) < 4) {
          sm[0] = m[0];
          sl[0] = l[0];
#pragma unroll
          for (int d = 0; d < DB; ++d) sacc[0][d] = acc[0][d];
        } else {
          fold<DB>(sm[0], sl[0], sacc[0], m[0], l[0], acc[0]);
        }
        m[0] = -INFINITY;
        l[0] = 0.f;
#pragma unroll
        for (int d = 0; d < DB; ++d) acc[0][d] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (SEQ && ((j & 31) == 31 || j + 1 == c.n_steps)) {
          // a super is complete as well: the same fold one level up
          if (j < 32) {
            tm = sm[0];
            tl = sl[0];
#pragma unroll
            for (int d = 0; d < DB; ++d) tacc[d] = sacc[0][d];
          } else {
            fold<DB>(tm, tl, tacc, sm[0], sl[0], sacc[0]);
          }
        }
      }
      entry_done();
    }
    // -- partial of this unit for every row that reaches into it
    if (SEQ) {
      if (qpos[0] >= 0) store_output<HD>(attn_out, d_attn, c.s, c.kvh, group, window, row[0], g, tacc, tl);
    } else if (SUPER && attn_out) {   // one unit per sequence: no partial, no merge pass
      if (qpos[0] >= 0)
        store_output<HD>(attn_out, d_attn, c.s, c.kvh, group, window, row[0], g, FOLD ? sacc[0] : acc[0], FOLD ? sl[0] : l[0]);
    } else if (qpos[0] >= c.k_lo) {
      const size_t prow = (((size_t)c.s * n_kv_heads + c.kvh) * n_units + c.unit) * r_pad + row[0];
      float* pa = part_acc + prow * HD;
#pragma unroll
      for (int d = 0; d < DB; ++d) *(f32x4*)(pa + d * 16 + g * 4) = SUPER && FOLD ? sacc[0][d] : acc[0][d];
      if (g == 0)
        *(float2*)(part_ml + prow * 2) = SUPER && FOLD ? make_float2(sm[0], sl[0]) : make_float2(m[0], l[0]);
    }
    c = c_next;
  }
  fetch_wait<0>();                      // the dummy fetches too
}

// The work items of a call: every (sequence, unit) pair that holds keys, as (s, unit, L, n), sorted
// by the number of 64-key steps it takes, longest first (the attention kernels deal them out in that
// order, which keeps the tail of a launch short); and the per-layer queue counters.  The order
// inside a class of equal length is whatever the slot counter gives: it decides only which
// workgroup computes an item, never a bit of the result.  One workgroup; runs once per call.
//
// seq_unit_keys != 0: the call may run with whole sequences as items (one unit of seq_unit_keys keys
// per sequence) if they deal out evenly enough over seq_grid workgroups (seq_per_item workgroups per
// item, dealt as the stream kernel deals them); the kernel lists them, adds up every workgroup's
// entries, and keeps that list (*seq_mode = 1) if the busiest workgroup has at most 5 % more than the
// average - else (*seq_mode = 0) it lists the units of unit_keys keys as usual.  The choice moves
// work between kernels that compute the same bits.
__global__ __launch_bounds__(256) void attention_plan_kernel(const int32_t* __restrict__ seq_len,
                                                             const int32_t* __restrict__ seq_n, int num_seqs,
                                                             int unit_keys, int seq_unit_keys, int seq_per_item,
                                                             int seq_grid, int4* __restrict__ items,
                                                             int32_t* __restrict__ item_count,
                                                             int32_t* __restrict__ queues, int n_layers,
                                                             int32_t* __restrict__ seq_mode) {
  // classes: an item's steps in units of class_steps, 1 .. nb <= MAXB (class_steps is 1 unless a unit is a whole sequence)
  constexpr int MAXB = SUPER_KEYS / STEP;
  __shared__ int count[MAXB + 1], cursor[MAXB + 1];
  __shared__ int n_items;
  __shared__ unsigned long long load_sum;
  __shared__ int load_max;
  for (int l = threadIdx.x; l < n_layers; l += 256) queues[l] = 0;
  auto list_items = [&](const int unit, const int class_steps) {
    const int nb = (unit / STEP + class_steps - 1) / class_steps;
    auto class_of = [&](int keys, int u) {
      return ((min(keys, (u + 1) * unit) - u * unit + STEP - 1) / STEP + class_steps - 1) / class_steps;
    };
    if (threadIdx.x <= MAXB) count[threadIdx.x] = 0;
    __syncthreads();
    for (int s = threadIdx.x; s < num_seqs; s += 256) {
      if (seq_len[s] < 0) continue;
      const int keys = seq_len[s] + seq_n[s];                // positions 0 .. keys-1 are attended to
      const int full = keys / unit;
      if (full) atomicAdd(&count[nb], full);
      if (keys % unit) atomicAdd(&count[class_of(keys, full)], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int at = 0;
      for (int c = nb; c >= 1; --c) {                        // longest class first
        cursor[c] = at;
        at += count[c];
      }
      n_items = at;
      *item_count = at;
    }
    __syncthreads();
    for (int s = threadIdx.x; s < num_seqs; s += 256) {
      if (seq_len[s] < 0) continue;
      const int L = seq_len[s], n = seq_n[s], keys = L + n;
      const int units = (keys + unit - 1) / unit;
      for (int u = 0; u < units; ++u) items[atomicAdd(&cursor[class_of(keys, u)], 1)] = make_int4(s, u, L, n);
    }
    __syncthreads();                                         // the list is complete (and visible to this workgroup)
  };
  int whole = 0;
  if (seq_unit_keys) {
    list_items(seq_unit_keys, (seq_unit_keys / STEP + MAXB - 1) / MAXB);
    if (threadIdx.x == 0) {
      load_sum = 0;
      load_max = 0;
    }
    __syncthreads();
    const int total = n_items * seq_per_item;
    for (int w = threadIdx.x; w < seq_grid; w += 256) {      // the entries workgroup w of the stream kernel would walk
      int load = 0;
      for (int ord = 0;; ++ord) {
        const int t = ord * seq_grid + ((ord & 1) ? seq_grid - 1 - w : w);
        if (t >= total) break;
        const int4 it = items[t / seq_per_item];
        load += (it.z + it.w + STEP - 1) / STEP + 1;
      }
      atomicAdd(&load_sum, (unsigned long long)load);
      atomicMax(&load_max, load);
    }
    __syncthreads();
    whole = (unsigned long long)load_max * seq_grid * 100ull <= load_sum * 105ull ? 1 : 0;
    __syncthreads();
  }
  if (!whole) list_items(unit_keys, 1);
  if (threadIdx.x == 0) *seq_mode = whole;
}

// Fold the partials of every query row (chunks inside a super left to right, then the supers
// left to right) and write the normalised output, bf16, into the tile layout of the
// O-projection's activation operand.  One thread per (row, 4 features).
template <int HD, bool SUPER>
__global__ void attention_merge_kernel(const float* __restrict__ part_acc, const float* __restrict__ part_ml,
                                       const int32_t* __restrict__ seq_len, const int32_t* __restrict__ seq_n,
                                       int n_kv_heads, int group, int window, int r_pad, int n_units, int d_attn,
                                       uint16_t* __restrict__ out, const int32_t* __restrict__ seq_mode) {
  if (*seq_mode) return;                // the attention kernel took whole sequences and wrote the output itself
  constexpr int QUADS = HD / 4;
  const int quad = threadIdx.x % QUADS;
  const int r = blockIdx.y * (blockDim.x / QUADS) + threadIdx.x / QUADS;   // (pairs can outnumber what grid.y allows)
  const int s = blockIdx.x / n_kv_heads, kvh = blockIdx.x % n_kv_heads;
  if (r >= group * window) return;
  const int L = seq_len[s], n = seq_n[s];
  const int i = r % window, hq = kvh * group + r / window;
  uint2* dst = (uint2*)(out + pk_off(s * window + i, hq * HD + quad * 4, d_attn));
  if (L < 0 || i >= n) {
    *dst = make_uint2(0, 0);
    return;
  }
  const size_t base = ((size_t)s * n_kv_heads + kvh) * n_units;
  auto slot_ml = [&](int u) { return *(const float2*)(part_ml + ((base + u) * r_pad + r) * 2); };
  auto slot_acc = [&](int u) { return *(const f32x4*)(part_acc + ((base + u) * r_pad + r) * HD + quad * 4); };
  float M, Ls;
  f32x4 A[1];
  if (SUPER) {
    const int last = (L + i) / SUPER_KEYS;
    float2 ml = slot_ml(0);
    M = ml.x;
    Ls = ml.y;
    A[0] = slot_acc(0);
    for (int u = 1; u <= last; ++u) {
      ml = slot_ml(u);
      const f32x4 B[1] = {slot_acc(u)};
      fold<1>(M, Ls, A, ml.x, ml.y, B);
    }
  } else {
    constexpr int PER = SUPER_KEYS / CHUNK;
    const int last = (L + i) / CHUNK;
    M = 0.f;
    Ls = 0.f;
    A[0] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 <= last; c0 += PER) {
      float2 ml = slot_ml(c0);
      float m2 = ml.x, l2 = ml.y;
      f32x4 a2[1] = {slot_acc(c0)};
      for (int c = c0 + 1; c <= min(c0 + PER - 1, last); ++c) {
        ml = slot_ml(c);
        const f32x4 B[1] = {slot_acc(c)};
        fold<1>(m2, l2, a2, ml.x, ml.y, B);
      }
      if (c0 == 0) {
        M = m2;
        Ls = l2;
        A[0] = a2[0];
      } else {
        fold<1>(M, Ls, A, m2, l2, a2);
      }
    }
  }
  uint2 o;
  o.x = pack2_bf16(A[0][0] / Ls, A[0][1] / Ls);
  o.y = pack2_bf16(A[0][2] / Ls, A[0][3] / Ls);
  *dst = o;
}

template <int HD, int CB, int NW, bool SUPER>
void launch_one(const llm42_model* m, int layer, const uint16_t* kp, const uint16_t* vp, const llm42_kv_cache* kv,
                int num_seqs, int window, const Workspace& ws, hipStream_t st) {
  const llm42_config& c = m->cfg;
  const float scale_log2 = (1.0f / sqrtf((float)c.head_dim)) * 1.44269504088896340736f;
  const int col_blocks = ws.r_pad / 16;
  const int y_blocks = (col_blocks + NW * CB - 1) / (NW * CB);
  // one workgroup per CU (the KV ring takes 128 KiB of LDS at head_dim 128), but no more than there can be items
  const long long max_items = (long long)num_seqs * ws.attn_units * c.n_kv_heads * y_blocks;
  const unsigned grid = (unsigned)std::min<long long>(m->num_cus * (HD == 128 ? 1 : 2), max_items);
  attention_kernel<HD, CB, NW, SUPER><<<grid, NW * 64, 0, st>>>(
      ws.q, (const uint4*)kp, (const uint4*)vp, kv->block_table, ws.seq_len, ws.seq_n, ws.attn_items, ws.attn_ctrl,
      ws.attn_ctrl + 1 + layer, c.n_kv_heads, m->group, window, ws.r_pad, y_blocks, kv->max_blocks_per_seq,
      ws.attn_units, scale_log2, ws.part_acc, ws.part_ml, SUPER && ws.attn_direct ? ws.attn : nullptr, m->d_attn);
  if (SUPER && ws.attn_direct) return;
  const int rows = m->group * window, rows_per_block = 256 / (HD / 4);
  attention_merge_kernel<HD, SUPER><<<dim3(num_seqs * c.n_kv_heads, (rows + rows_per_block - 1) / rows_per_block), 256,
                                      0, st>>>(ws.part_acc, ws.part_ml, ws.seq_len, ws.seq_n, c.n_kv_heads, m->group,
                                               window, ws.r_pad, ws.attn_units, m->d_attn, ws.attn,
                                               ws.attn_ctrl + 1 + c.n_layers);
}

// Workgroups of a stream-kernel launch: one per CU at head_dim 128 (two at 64), no more than there are items.
long long stream_grid(const llm42_model* m, int num_seqs, int units, int r_pad) {
  const long long max_items = (long long)num_seqs * units * m->cfg.n_kv_heads * ((r_pad / 16 + 7) / 8);
  return std::min<long long>(m->num_cus * (m->cfg.head_dim == 128 ? 1 : 2), max_items);
}

template <int HD, bool SUPER, bool FOLD, bool SEQ = false>
void launch_stream(const llm42_model* m, const uint16_t* kp, const uint16_t* vp, const llm42_kv_cache* kv, int num_seqs,
                   int window, const Workspace& ws, hipStream_t st) {
  const llm42_config& c = m->cfg;
  const float scale_log2 = (1.0f / sqrtf((float)c.head_dim)) * 1.44269504088896340736f;
  const int y_blocks = (ws.r_pad / 16 + 7) / 8;
  const unsigned grid = (unsigned)stream_grid(m, num_seqs, SEQ ? 1 : ws.attn_units, ws.r_pad);
  attention_stream_kernel<HD, SUPER, FOLD, SEQ><<<grid, 512, 0, st>>>(
      ws.q, (const uint4*)kp, (const uint4*)vp, kv->block_table, ws.attn_items, ws.attn_ctrl, c.n_kv_heads, m->group,
      window, ws.r_pad, y_blocks, kv->max_blocks_per_seq, ws.attn_units, scale_log2, ws.part_acc, ws.part_ml,
      SEQ || (SUPER && ws.attn_direct) ? ws.attn : nullptr, m->d_attn, ws.attn_ctrl + 1 + c.n_layers);
  if (SEQ || (SUPER && ws.attn_direct)) return;
  const int rows = m->group * window, rows_per_block = 256 / (HD / 4);
  attention_merge_kernel<HD, SUPER><<<dim3(num_seqs * c.n_kv_heads, (rows + rows_per_block - 1) / rows_per_block), 256,
                                      0, st>>>(ws.part_acc, ws.part_ml, ws.seq_len, ws.seq_n, c.n_kv_heads, m->group,
                                               window, ws.r_pad, ws.attn_units, m->d_attn, ws.attn,
                                               ws.attn_ctrl + 1 + c.n_layers);
}

template <int HD>
void launch_hd(const llm42_model* m, int layer, const uint16_t* kp, const uint16_t* vp, const llm42_kv_cache* kv,
               int num_seqs, int window, const Workspace& ws, hipStream_t st) {
  // 8 row blocks or more per (sequence, kv head): 8 waves of one row block each, two per SIMD, so
  // that one wave's MFMAs run under the other's softmax arithmetic, as one stream per CU; fewer: 4 waves.
  const bool wide = ws.r_pad / 16 >= 8;
  // (a call that may take whole sequences as items launches that kernel too; the plan's choice, made on the device
  // from the lengths, leaves one of the two with nothing to do)
  if (ws.attn_seq) launch_stream<HD, true, true, true>(m, kp, vp, kv, num_seqs, window, ws, st);
  if (ws.attn_super) {
    if (wide && ws.batch_chosen) launch_stream<HD, true, false>(m, kp, vp, kv, num_seqs, window, ws, st);
    else if (wide) launch_stream<HD, true, true>(m, kp, vp, kv, num_seqs, window, ws, st);
    else launch_one<HD, 1, 4, true>(m, layer, kp, vp, kv, num_seqs, window, ws, st);
  } else {
    if (wide) launch_stream<HD, false, true>(m, kp, vp, kv, num_seqs, window, ws, st);
    else launch_one<HD, 1, 4, false>(m, layer, kp, vp, kv, num_seqs, window, ws, st);
  }
}

}  // namespace

void launch_attention_plan(const llm42_model* m, int num_seqs, int max_context, const Workspace& ws, hipStream_t st) {
  // as a whole-sequence item a unit has as many keys as the longest sequence of the call may have
  const int seq_unit_keys = ws.attn_seq ? (max_context + STEP - 1) / STEP * STEP : 0;
  const int seq_per_item = m->cfg.n_kv_heads * ((ws.r_pad / 16 + 7) / 8);
  attention_plan_kernel<<<1, 256, 0, st>>>(ws.seq_len, ws.seq_n, num_seqs, ws.attn_super ? SUPER_KEYS : CHUNK,
                                           seq_unit_keys, seq_per_item, (int)stream_grid(m, num_seqs, 1, ws.r_pad),
                                           ws.attn_items, ws.attn_ctrl, ws.attn_ctrl + 1, m->cfg.n_layers,
                                           ws.attn_ctrl + 1 + m->cfg.n_layers);
}

int attention_units(bool super_mode, int max_context) {
  const int keys = super_mode ? SUPER_KEYS : CHUNK;
  return (max_context + keys - 1) / keys;
}

void launch_attention(const llm42_model* m, int layer, const llm42_kv_cache* kv, int num_seqs, int window,
                      int max_context, const Workspace& ws, hipStream_t st) {
  const llm42_config& c = m->cfg;
  const size_t plane = (size_t)kv->num_blocks * c.n_kv_heads * 16 * c.head_dim;
  const uint16_t* kp = (const uint16_t*)kv->kv_base + ((size_t)layer * 2 + 0) * plane;
  const uint16_t* vp = (const uint16_t*)kv->kv_base + ((size_t)layer * 2 + 1) * plane;
  if (c.head_dim == 128) launch_hd<128>(m, layer, kp, vp, kv, num_seqs, window, ws, st);
  else launch_hd<64>(m, layer, kp, vp, kv, num_seqs, window, ws, st);
}
