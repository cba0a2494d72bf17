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
// Work distribution (free to change, does not touch the bits): a workgroup of 4
// waves owns one unit of keys - a chunk (few sequences: more parallelism, chunk
// partials are written and merge_kernel does all folds) or a whole super (many
// sequences: chunk partials are folded in registers, 8 times fewer partials go
// through HBM) - for up to 8 blocks of 16 query rows of one (sequence, kv head);
// query rows are ordered r = q_head_in_group * window + i.  K and V tiles are
// fetched once per workgroup, 128 keys at a time (the next stage's loads are issued
// before the current stage is computed), double buffered through LDS in MFMA operand order (see the KV tile layouts in llm42.h), so no transpose is needed.
#include "llm42_dev.h"

namespace {

constexpr int STEP = 64, CHUNK = 256, SUPER_KEYS = 2048, STAGE = 128;

union Frag {
  bf16x8 v;
  uint4 u;
  uint2 h[2];
};

// state <- state (+) part, the only way two partials are ever combined.
template <int NV>
__device__ inline void fold(float& M, float& L, f32x4 (&A)[NV], float m2, float l2, const f32x4 (&a2)[NV]) {
  const float mn = fmaxf(M, m2);
  const float mu = mn == -INFINITY ? 0.f : mn;
  const float a = __builtin_amdgcn_exp2f(M - mu), b = __builtin_amdgcn_exp2f(m2 - mu);
  L = L * a + l2 * b;
#pragma unroll
  for (int i = 0; i < NV; ++i) A[i] = A[i] * a + a2[i] * b;
  M = mn;
}

// A lane's share of one KV tile in flight between global memory and LDS: TL pieces of 16 bytes.
// (Native vector type on purpose: register arrays of HIP_vector_type structs end up in scratch.)
template <int TL>
__device__ __forceinline__ void tile_load(bf16x8 (&r)[TL], const uint4* src) {
#pragma unroll
  for (int i = 0; i < TL; ++i) r[i] = ((const bf16x8*)src)[i * 64];
}
template <int TL>
__device__ __forceinline__ void tile_store(uint4* dst, const bf16x8 (&r)[TL]) {
#pragma unroll
  for (int i = 0; i < TL; ++i) ((bf16x8*)dst)[i * 64] = r[i];
}

template <int HD, int CB, bool SUPER>
__global__ __launch_bounds__(256) void attention_kernel(
    const uint16_t* __restrict__ q, const uint4* __restrict__ k_plane, const uint4* __restrict__ v_plane,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_len, const int32_t* __restrict__ seq_n,
    int n_kv_heads, int group, int window, int r_pad, int max_blocks_per_seq, int n_units, float scale_log2,
    float* __restrict__ part_acc, float* __restrict__ part_ml) {
  constexpr int DK = HD / 32;        // MFMA k-steps over the head dimension (scores)
  constexpr int DB = HD / 16;        // 16-feature blocks of the output
  constexpr int TV4 = HD * 2;        // uint4 per KV tile (16 tokens x HD bf16)
  constexpr int TL = TV4 / 64;       // uint4 per lane per tile
  constexpr int UNIT = SUPER ? SUPER_KEYS : CHUNK;
  __shared__ uint4 lds_k[2][8 * TV4];
  __shared__ uint4 lds_v[2][8 * TV4];
  __shared__ int wg_max[4];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const int unit = blockIdx.x;
  const int s = blockIdx.z / n_kv_heads, kvh = blockIdx.z % n_kv_heads;
  const int k_lo = unit * UNIT;
  const int32_t* bt = block_table + (size_t)s * max_blocks_per_seq;
  // Requested before anything is known about the sequence, so that the three latencies (lengths,
  // block ids, query operands) overlap: the unit's block-table entries (clamped to the table, not
  // yet to the sequence) and the query operands of this wave's row blocks.
  const int first_blk = k_lo >> 4;
  const int raw0 = bt[min(first_blk + lane, max_blocks_per_seq - 1)];
  const int raw1 = SUPER ? bt[min(first_blk + 64 + lane, max_blocks_per_seq - 1)] : 0;
  Frag qf[CB][DK];
  int row[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    row[cb] = ((blockIdx.y * 4 + wave) * CB + cb) * 16 + col;
    // row blocks past r_pad (grid padding) read the last real block instead; their rows are dead anyway
    const int rb = min(row[cb] >> 4, r_pad / 16 - 1);
    const uint16_t* qb = q + ((size_t)s * n_kv_heads + kvh) * r_pad * HD + (size_t)rb * DK * 512;
#pragma unroll
    for (int d = 0; d < DK; ++d) qf[cb][d].u = *(const uint4*)(qb + d * 512 + lane * 8);
  }
  const int L = seq_len[s], n = seq_n[s];
  if (L < 0) return;                                         // whole workgroup

  int qpos[CB];
  int wmax = -1;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int i = row[cb] % window;
    qpos[cb] = (row[cb] < group * window && i < n) ? L + i : -1;
    wmax = max(wmax, qpos[cb]);
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) wmax = max(wmax, __shfl_xor(wmax, off));
  if (lane == 0) wg_max[wave] = wmax;
  __syncthreads();
  const int gmax = max(max(wg_max[0], wg_max[1]), max(wg_max[2], wg_max[3]));
  if (gmax < k_lo) return;                                   // whole workgroup: nobody looks into this unit
  const int k_hi = min(gmax + 1, k_lo + UNIT);               // exclusive; <= L + n
  const int n_stages = (k_hi - k_lo + STAGE - 1) / STAGE;
  const int last_blk = (k_hi - 1) >> 4;
  // table entries past the last needed block may hold anything: replace them by the last needed
  // block's id (its data is fetched in their place, and every key in those positions is masked)
  const int last_id = __shfl((last_blk - first_blk) < 64 ? raw0 : raw1, (last_blk - first_blk) & 63);
  const int ids0 = first_blk + lane <= last_blk ? raw0 : last_id;
  const int ids1 = first_blk + 64 + lane <= last_blk ? raw1 : last_id;

  // each wave fetches two of the eight blocks of a stage into registers (issued before the current
  // stage is computed) and parks them in the other LDS buffer afterwards
  bf16x8 kreg0[TL], kreg1[TL], vreg0[TL], vreg1[TL];
#define ATT_FETCH(st_)                                                                         \
  do {                                                                                         \
    const int bj_ = (st_) * 8 + wave * 2;               /* block index inside the unit */      \
    const int id0_ = __shfl(bj_ < 64 ? ids0 : ids1, bj_ & 63);                                 \
    const int id1_ = __shfl(bj_ + 1 < 64 ? ids0 : ids1, (bj_ + 1) & 63);                       \
    tile_load<TL>(kreg0, k_plane + ((size_t)id0_ * n_kv_heads + kvh) * TV4 + lane);            \
    tile_load<TL>(vreg0, v_plane + ((size_t)id0_ * n_kv_heads + kvh) * TV4 + lane);            \
    tile_load<TL>(kreg1, k_plane + ((size_t)id1_ * n_kv_heads + kvh) * TV4 + lane);            \
    tile_load<TL>(vreg1, v_plane + ((size_t)id1_ * n_kv_heads + kvh) * TV4 + lane);            \
  } while (0)
#define ATT_PARK(buf_)                                                                         \
  do {                                                                                         \
    tile_store<TL>(&lds_k[buf_][(wave * 2) * TV4 + lane], kreg0);                              \
    tile_store<TL>(&lds_v[buf_][(wave * 2) * TV4 + lane], vreg0);                              \
    tile_store<TL>(&lds_k[buf_][(wave * 2 + 1) * TV4 + lane], kreg1);                          \
    tile_store<TL>(&lds_v[buf_][(wave * 2 + 1) * TV4 + lane], vreg1);                          \
  } while (0)

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

  ATT_FETCH(0);
  ATT_PARK(0);
  __syncthreads();
  for (int st = 0; st < n_stages; ++st) {
    const int buf = st & 1;
    if (st + 1 < n_stages) ATT_FETCH(st + 1);
    const uint16_t* vbase = (const uint16_t*)lds_v[buf];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int k0 = k_lo + st * STAGE + s2 * STEP;
      if (k0 >= k_hi) break;                                  // workgroup-uniform
      // ---- scores of 4 blocks of 16 keys: S^T[key][query] ---------------------------------
      f32x4 sc[CB][4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) sc[cb][b] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (k0 + b * 16 < k_hi) {                            // workgroup-uniform
#pragma unroll
          for (int d = 0; d < DK; ++d) {
            Frag kf;
            kf.u = lds_k[buf][(s2 * 4 + b) * TV4 + d * 64 + lane];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) sc[cb][b] = mfma16(kf.v, qf[cb][d].v, sc[cb][b]);
          }
        }
      }
      // ---- mask, online softmax state, P in bf16 ------------------------------------------
      Frag pf[CB][2];
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        float mx = -INFINITY;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int kpos = k0 + b * 16 + g * 4 + e;
            const float v = kpos <= qpos[cb] ? sc[cb][b][e] * scale_log2 : -INFINITY;
            sc[cb][b][e] = v;
            mx = fmaxf(mx, v);
          }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m[cb], mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m[cb] - m_use);
        float rs = 0.f;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
          for (int e = 0; e < 4; ++e) sc[cb][b][e] = __builtin_amdgcn_exp2f(sc[cb][b][e] - m_use);
          rs += ((sc[cb][b][0] + sc[cb][b][1]) + sc[cb][b][2]) + sc[cb][b][3];
        }
        rs += __shfl_xor(rs, 16);
        rs += __shfl_xor(rs, 32);
        l[cb] = l[cb] * alpha + rs;
        m[cb] = m_new;
#pragma unroll
        for (int d = 0; d < DB; ++d) acc[cb][d] *= alpha;
        // k-slot e of lane group g is key g*4+e of the first block of a pair (e < 4) or of the
        // second (e >= 4); V below uses the same assignment
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          pf[cb][kk].h[0].x = pack2_bf16(sc[cb][2 * kk][0], sc[cb][2 * kk][1]);
          pf[cb][kk].h[0].y = pack2_bf16(sc[cb][2 * kk][2], sc[cb][2 * kk][3]);
          pf[cb][kk].h[1].x = pack2_bf16(sc[cb][2 * kk + 1][0], sc[cb][2 * kk + 1][1]);
          pf[cb][kk].h[1].y = pack2_bf16(sc[cb][2 * kk + 1][2], sc[cb][2 * kk + 1][3]);
        }
      }
      // ---- acc^T[feature][query] += V^T P^T, 32 keys per MFMA ------------------------------
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const int kp0 = k0 + kk * 32 + g * 4, kp1 = kp0 + 16;
        if (k0 + kk * 32 >= k_hi) break;                      // workgroup-uniform
        const uint16_t* vt0 = vbase + (size_t)(s2 * 4 + 2 * kk) * TV4 * 8;
        const uint16_t* vt1 = vt0 + TV4 * 8;
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          Frag vf;
          vf.h[0] = *(const uint2*)(vt0 + (d * 16 + col) * 16 + g * 4);
          vf.h[1] = *(const uint2*)(vt1 + (d * 16 + col) * 16 + g * 4);
          // slots at or beyond k_hi hold stale, never-written or foreign data: force them to zero
          // so that 0 * garbage cannot produce a NaN
          if (kp0 + 3 >= k_hi) {
            if (kp0 + 0 >= k_hi) vf.h[0].x &= 0xFFFF0000u;
            if (kp0 + 1 >= k_hi) vf.h[0].x &= 0x0000FFFFu;
            if (kp0 + 2 >= k_hi) vf.h[0].y &= 0xFFFF0000u;
            if (kp0 + 3 >= k_hi) vf.h[0].y &= 0x0000FFFFu;
          }
          if (kp1 + 3 >= k_hi) {
            if (kp1 + 0 >= k_hi) vf.h[1].x &= 0xFFFF0000u;
            if (kp1 + 1 >= k_hi) vf.h[1].x &= 0x0000FFFFu;
            if (kp1 + 2 >= k_hi) vf.h[1].y &= 0xFFFF0000u;
            if (kp1 + 3 >= k_hi) vf.h[1].y &= 0x0000FFFFu;
          }
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) acc[cb][d] = mfma16(vf.v, pf[cb][kk].v, acc[cb][d]);
        }
      }
    }
    if (SUPER && ((st & 1) || st + 1 == n_stages)) {
      // a chunk is complete: fold it into the running super partial and start the next one afresh
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        if (st < 2) {
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
    if (st + 1 < n_stages) ATT_PARK(buf ^ 1);
    __syncthreads();
  }

  // ---- partial of this unit for every row that reaches into it ---------------------------------
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    if (qpos[cb] < k_lo) continue;
    const size_t prow = (((size_t)s * n_kv_heads + kvh) * n_units + unit) * r_pad + row[cb];
    float* pa = part_acc + prow * HD;
#pragma unroll
    for (int d = 0; d < DB; ++d) *(f32x4*)(pa + d * 16 + g * 4) = SUPER ? sacc[cb][d] : acc[cb][d];
    if (g == 0) *(float2*)(part_ml + prow * 2) = SUPER ? make_float2(sm[cb], sl[cb]) : make_float2(m[cb], l[cb]);
  }
}

#undef ATT_FETCH
#undef ATT_PARK

// Fold the partials of every query row (chunks inside a super left to right, then the supers
// left to right) and write the normalised output, bf16, into the tile layout of the
// O-projection's activation operand.  One thread per (row, 4 features).
template <int HD, bool SUPER>
__global__ void attention_merge_kernel(const float* __restrict__ part_acc, const float* __restrict__ part_ml,
                                       const int32_t* __restrict__ seq_len, const int32_t* __restrict__ seq_n,
                                       int n_kv_heads, int group, int window, int r_pad, int n_units, int d_attn,
                                       uint16_t* __restrict__ out) {
  constexpr int QUADS = HD / 4;
  const int quad = threadIdx.x % QUADS;
  const int r = blockIdx.x * (blockDim.x / QUADS) + threadIdx.x / QUADS;
  const int s = blockIdx.y / n_kv_heads, kvh = blockIdx.y % n_kv_heads;
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

template <int HD, int CB, bool SUPER>
void launch_one(const llm42_model* m, const uint16_t* kp, const uint16_t* vp, const llm42_kv_cache* kv, int num_seqs,
                int window, const Workspace& ws, hipStream_t st) {
  const llm42_config& c = m->cfg;
  const float scale_log2 = (1.0f / sqrtf((float)c.head_dim)) * 1.44269504088896340736f;
  const int col_blocks = ws.r_pad / 16;
  const dim3 grid(ws.attn_units, (col_blocks + 4 * CB - 1) / (4 * CB), num_seqs * c.n_kv_heads);
  attention_kernel<HD, CB, SUPER><<<grid, 256, 0, st>>>(ws.q, (const uint4*)kp, (const uint4*)vp, kv->block_table,
                                                        ws.seq_len, ws.seq_n, c.n_kv_heads, m->group, window, ws.r_pad,
                                                        kv->max_blocks_per_seq, ws.attn_units, scale_log2, ws.part_acc,
                                                        ws.part_ml);
  const int rows = m->group * window, rows_per_block = 256 / (HD / 4);
  attention_merge_kernel<HD, SUPER><<<dim3((rows + rows_per_block - 1) / rows_per_block, num_seqs * c.n_kv_heads), 256,
                                      0, st>>>(ws.part_acc, ws.part_ml, ws.seq_len, ws.seq_n, c.n_kv_heads, m->group,
                                               window, ws.r_pad, ws.attn_units, m->d_attn, ws.attn);
}

template <int HD>
void launch_hd(const llm42_model* m, const uint16_t* kp, const uint16_t* vp, const llm42_kv_cache* kv, int num_seqs,
               int window, const Workspace& ws, hipStream_t st) {
  const bool two = ws.r_pad / 16 >= 8;
  if (ws.attn_super) {
    if (two) launch_one<HD, 2, true>(m, kp, vp, kv, num_seqs, window, ws, st);
    else launch_one<HD, 1, true>(m, kp, vp, kv, num_seqs, window, ws, st);
  } else {
    if (two) launch_one<HD, 2, false>(m, kp, vp, kv, num_seqs, window, ws, st);
    else launch_one<HD, 1, false>(m, kp, vp, kv, num_seqs, window, ws, st);
  }
}

}  // namespace

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
  if (c.head_dim == 128) launch_hd<128>(m, kp, vp, kv, num_seqs, window, ws, st);
  else launch_hd<64>(m, kp, vp, kv, num_seqs, window, ws, st);
}
