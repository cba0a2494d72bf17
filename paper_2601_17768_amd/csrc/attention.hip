// Causal window attention over the paged KV cache (grouped-query), bf16 MFMA
// with fp32 online softmax.
//
// Reduction schedule of one query row at absolute position p (it depends on p
// and on nothing else - not on the window, the row's index in it, the batch, or
// the context lengths of other sequences):
//   * keys are cut at absolute positions into super-chunks of LLM42_SUPERCHUNK;
//     super-chunk c holds keys [c*SC, min((c+1)*SC, p+1));
//   * inside a super-chunk the state (m, l, acc) starts at (-inf, 0, 0) and is
//     advanced by online-softmax steps over LLM42_KEYSTEP keys in ascending
//     order (also cut at absolute positions); a step computes its scores with 4
//     MFMA k-steps per 16-key block, reduces max and sum over its 64 keys in a
//     fixed tree, rescales, and adds P V with two MFMA k-steps of 32 keys;
//   * the super-chunk partials are folded in ascending order (merge kernel).
// Keys beyond p contribute exact zeros (masked before the exponential) and a
// step in which every key of a row is masked leaves that row's state bit for bit
// unchanged, so rows of different positions can share a wave.
//
// Work distribution (free to change, does not touch the bits): one wave per
// (super-chunk, block of 16 query rows, sequence x kv head); the query rows of a
// kv head are ordered r = q_head_in_group * window + i.  K, V and Q operands are
// read straight from HBM/L2 in MFMA operand order (see the KV tile layouts in
// llm42.h), so no LDS transpose is needed.
#include "llm42_dev.h"

namespace {

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

union Frag {
  bf16x8 v;
  uint4 u;
  uint2 h[2];
};

template <int HD>
__global__ __launch_bounds__(256) void attention_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_plane, const uint16_t* __restrict__ v_plane,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_len, const int32_t* __restrict__ seq_n,
    int n_kv_heads, int group, int window, int r_pad, int max_blocks_per_seq, int n_super, float scale_log2,
    float* __restrict__ part_acc, float* __restrict__ part_ml) {
  constexpr int DK = HD / 32;   // MFMA k-steps over the head dimension (scores)
  constexpr int DB = HD / 16;   // 16-feature blocks of the output
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = blockIdx.x;
  const int cb = blockIdx.y * 4 + wave;
  const int s = blockIdx.z / n_kv_heads, kvh = blockIdx.z % n_kv_heads;
  if (cb * 16 >= r_pad) return;
  const int L = seq_len[s], n = seq_n[s];
  if (L < 0) return;
  const int col = lane & 15, g = lane >> 4;
  const int r = cb * 16 + col;
  const int i = r % window;
  const bool live = r < group * window && i < n;
  const int qpos = live ? L + i : -1;
  const int k_begin = c * LLM42_SUPERCHUNK;
  // last position any row of this wave may look at
  int wave_max = qpos;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) wave_max = max(wave_max, __shfl_xor(wave_max, off));
  if (wave_max < k_begin) return;
  const int k_end = min(wave_max + 1, k_begin + LLM42_SUPERCHUNK);   // exclusive
  const int total = L + n;                                          // first position that holds garbage

  const uint16_t* qbase = q + ((size_t)s * n_kv_heads + kvh) * r_pad * HD + (size_t)cb * DK * 512;
  Frag qf[DK];
#pragma unroll
  for (int d = 0; d < DK; ++d) qf[d].u = *(const uint4*)(qbase + d * 512 + lane * 8);

  float m = -INFINITY, l = 0.f;
  f32x4 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) acc[d] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const int32_t* bt = block_table + (size_t)s * max_blocks_per_seq;

  for (int k0 = k_begin; k0 < k_end; k0 += LLM42_KEYSTEP) {
    // ---- scores of 4 blocks of 16 keys: S^T[key][query] -------------------------------
    f32x4 sc[4];
    int blk[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int kb0 = k0 + b * 16;
      sc[b] = (f32x4){0.f, 0.f, 0.f, 0.f};
      blk[b] = -1;
      if (kb0 < k_end) {   // wave-uniform
        blk[b] = bt[kb0 >> 4];
        const uint16_t* kt = k_plane + ((size_t)blk[b] * n_kv_heads + kvh) * 16 * HD;
#pragma unroll
        for (int d = 0; d < DK; ++d) {
          Frag kf;
          kf.u = *(const uint4*)(kt + d * 512 + lane * 8);
          sc[b] = mfma16(kf.v, qf[d].v, sc[b]);
        }
      }
    }
    // ---- mask, running max -------------------------------------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int kpos = k0 + b * 16 + g * 4 + e;
        const float v = kpos <= qpos ? sc[b][e] * scale_log2 : -INFINITY;
        sc[b][e] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_use);
    // ---- exponentials, row sum in a fixed tree ----------------------------------------
    float rs = 0.f;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
#pragma unroll
      for (int e = 0; e < 4; ++e) sc[b][e] = __builtin_amdgcn_exp2f(sc[b][e] - m_use);
      rs += ((sc[b][0] + sc[b][1]) + sc[b][2]) + sc[b][3];
    }
    rs += __shfl_xor(rs, 16);
    rs += __shfl_xor(rs, 32);
    l = l * alpha + rs;
    m = m_new;
#pragma unroll
    for (int d = 0; d < DB; ++d) acc[d] *= alpha;
    // ---- acc^T[feature][query] += V^T P^T, 32 keys per MFMA ----------------------------
    // k-slot e of lane group g is key g*4+e of the first block (e < 4) or of the second (e >= 4);
    // P and V use the same assignment.
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      if (blk[2 * kk] < 0) continue;   // wave-uniform: both blocks beyond k_end
      Frag pf;
      pf.h[0].x = pack2_bf16(sc[2 * kk][0], sc[2 * kk][1]);
      pf.h[0].y = pack2_bf16(sc[2 * kk][2], sc[2 * kk][3]);
      pf.h[1].x = pack2_bf16(sc[2 * kk + 1][0], sc[2 * kk + 1][1]);
      pf.h[1].y = pack2_bf16(sc[2 * kk + 1][2], sc[2 * kk + 1][3]);
      const uint16_t* vt0 = v_plane + ((size_t)blk[2 * kk] * n_kv_heads + kvh) * 16 * HD;
      const bool has1 = blk[2 * kk + 1] >= 0;
      const uint16_t* vt1 = v_plane + ((size_t)(has1 ? blk[2 * kk + 1] : blk[2 * kk]) * n_kv_heads + kvh) * 16 * HD;
      // slots at or beyond `total` hold stale or never-written data: force them to zero so that
      // 0 * garbage cannot produce a NaN
      const int kp0 = k0 + kk * 32 + g * 4, kp1 = kp0 + 16;
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        Frag vf;
        vf.h[0] = *(const uint2*)(vt0 + (d * 16 + col) * 16 + g * 4);
        vf.h[1] = has1 ? *(const uint2*)(vt1 + (d * 16 + col) * 16 + g * 4) : make_uint2(0, 0);
        if (kp0 + 3 >= total) {
          if (kp0 + 0 >= total) vf.h[0].x &= 0xFFFF0000u;
          if (kp0 + 1 >= total) vf.h[0].x &= 0x0000FFFFu;
          if (kp0 + 2 >= total) vf.h[0].y &= 0xFFFF0000u;
          if (kp0 + 3 >= total) vf.h[0].y &= 0x0000FFFFu;
        }
        if (kp1 + 3 >= total) {
          if (kp1 + 0 >= total) vf.h[1].x &= 0xFFFF0000u;
          if (kp1 + 1 >= total) vf.h[1].x &= 0x0000FFFFu;
          if (kp1 + 2 >= total) vf.h[1].y &= 0xFFFF0000u;
          if (kp1 + 3 >= total) vf.h[1].y &= 0x0000FFFFu;
        }
        acc[d] = mfma16(vf.v, pf.v, acc[d]);
      }
    }
  }

  // ---- partial (m, l, acc) of this super-chunk for every row that reaches into it ------
  if (qpos >= k_begin) {
    const size_t prow = (((size_t)s * n_kv_heads + kvh) * n_super + c) * r_pad + r;
    float* pa = part_acc + prow * HD;
#pragma unroll
    for (int d = 0; d < DB; ++d) *(f32x4*)(pa + d * 16 + g * 4) = acc[d];
    if (g == 0) *(float2*)(part_ml + prow * 2) = make_float2(m, l);
  }
}

// Fold the super-chunk partials of every query row in ascending order and write
// the normalised output, bf16, into the tile layout of the O-projection's
// activation operand.  One thread per (row, 4 features).
template <int HD>
__global__ void attention_merge_kernel(const float* __restrict__ part_acc, const float* __restrict__ part_ml,
                                       const int32_t* __restrict__ seq_len, const int32_t* __restrict__ seq_n,
                                       int n_kv_heads, int group, int window, int r_pad, int n_super, int d_attn,
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
  const int last = (L + i) / LLM42_SUPERCHUNK;
  const size_t base = ((size_t)s * n_kv_heads + kvh) * n_super;
  size_t prow = base * r_pad + r;
  float2 ml = *(const float2*)(part_ml + prow * 2);
  float M = ml.x, Ls = ml.y;
  f32x4 A = *(const f32x4*)(part_acc + prow * HD + quad * 4);
  for (int c = 1; c <= last; ++c) {
    prow = (base + c) * r_pad + r;
    ml = *(const float2*)(part_ml + prow * 2);
    const f32x4 B = *(const f32x4*)(part_acc + prow * HD + quad * 4);
    const float mn = fmaxf(M, ml.x);
    const float a = __builtin_amdgcn_exp2f(M - mn), b = __builtin_amdgcn_exp2f(ml.x - mn);
    Ls = Ls * a + ml.y * b;
    A = A * a + B * b;
    M = mn;
  }
  uint2 o;
  o.x = pack2_bf16(A[0] / Ls, A[1] / Ls);
  o.y = pack2_bf16(A[2] / Ls, A[3] / Ls);
  *dst = o;
}

}  // namespace

void launch_attention(const llm42_model* m, int layer, const llm42_kv_cache* kv, int num_seqs, int window,
                      int max_context, const Workspace& ws, hipStream_t st) {
  const llm42_config& c = m->cfg;
  const size_t plane = (size_t)kv->num_blocks * c.n_kv_heads * 16 * c.head_dim;
  const uint16_t* kp = (const uint16_t*)kv->kv_base + ((size_t)layer * 2 + 0) * plane;
  const uint16_t* vp = (const uint16_t*)kv->kv_base + ((size_t)layer * 2 + 1) * plane;
  const float scale_log2 = (1.0f / sqrtf((float)c.head_dim)) * 1.44269504088896340736f;
  const int n_super = (max_context + LLM42_SUPERCHUNK - 1) / LLM42_SUPERCHUNK;   // == ws.n_super
  const dim3 grid(n_super, (ws.r_pad / 16 + 3) / 4, num_seqs * c.n_kv_heads);
  const int rows = m->group * window;
  if (c.head_dim == 128) {
    attention_kernel<128><<<grid, 256, 0, st>>>(ws.q, kp, vp, kv->block_table, ws.seq_len, ws.seq_n, c.n_kv_heads,
                                                m->group, window, ws.r_pad, kv->max_blocks_per_seq, ws.n_super,
                                                scale_log2, ws.part_acc, ws.part_ml);
    const int rows_per_block = 256 / 32;
    attention_merge_kernel<128><<<dim3((rows + rows_per_block - 1) / rows_per_block, num_seqs * c.n_kv_heads), 256,
                                  0, st>>>(ws.part_acc, ws.part_ml, ws.seq_len, ws.seq_n, c.n_kv_heads, m->group,
                                           window, ws.r_pad, ws.n_super, m->d_attn, ws.attn);
  } else {
    attention_kernel<64><<<grid, 256, 0, st>>>(ws.q, kp, vp, kv->block_table, ws.seq_len, ws.seq_n, c.n_kv_heads,
                                               m->group, window, ws.r_pad, kv->max_blocks_per_seq, ws.n_super,
                                               scale_log2, ws.part_acc, ws.part_ml);
    const int rows_per_block = 256 / 16;
    attention_merge_kernel<64><<<dim3((rows + rows_per_block - 1) / rows_per_block, num_seqs * c.n_kv_heads), 256,
                                 0, st>>>(ws.part_acc, ws.part_ml, ws.seq_len, ws.seq_n, c.n_kv_heads, m->group,
                                          window, ws.r_pad, ws.n_super, m->d_attn, ws.attn);
  }
}
