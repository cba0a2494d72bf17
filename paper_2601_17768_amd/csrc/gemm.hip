// bf16 MFMA GEMMs of the verifier pass, D[feature][token] = sum_k W[feature][k] X[token][k],
// with the layer-specific epilogues fused (rotary embedding + KV-cache write,
// residual add, SwiGLU, logits + arg-max partials).
//
// Reduction schedule (what fixes the bits of every output element): one fp32
// accumulator per element, started at zero, updated by v_mfma_f32_16x16x32_bf16
// over k-tiles 0, 1, 2, ... in ascending order; no split along K.  The schedule
// depends on K only.  How many token blocks a wave owns, how many waves share a
// workgroup and how the grid is shaped are work-distribution choices that do not
// touch it, so they may change with the number of rows.
#include "llm42_dev.h"

namespace {

struct QkvEpi {
  const float2* rope;        // [max_position][head_dim/2] (cos, sin)
  const int32_t* row_pos;
  const int32_t* row_seq;
  const int32_t* block_table;
  uint16_t* q;               // [seq][kv head][r_pad][head_dim] tile layout, r = q-head-in-group * window + i
  uint16_t* k_plane;         // this layer's K tiles [block][kv head][16*head_dim]
  uint16_t* v_plane;
  int n_q_heads, n_kv_heads, head_dim, group, window, r_pad, max_blocks_per_seq;

  __device__ void operator()(int nb, int lane, int row, const f32x4 acc) const {
    const int pos = row_pos[row];
    if (pos < 0) return;
    const int blocks_per_head = head_dim >> 4;
    const int head = nb / blocks_per_head, t = nb % blocks_per_head, g = lane >> 4;
    const int j0 = t * 8 + g * 2;           // features j0, j0+1 and their rotary partners j0 + hd/2, j0+1 + hd/2
    const int half = head_dim >> 1;
    const int s = row_seq[row];
    float lo0 = acc[0], lo1 = acc[1], hi0 = acc[2], hi1 = acc[3];
    if (head < n_q_heads + n_kv_heads) {
      const float2 cs0 = rope[(size_t)pos * half + j0], cs1 = rope[(size_t)pos * half + j0 + 1];
      const float a0 = lo0 * cs0.x - hi0 * cs0.y, b0 = hi0 * cs0.x + lo0 * cs0.y;
      const float a1 = lo1 * cs1.x - hi1 * cs1.y, b1 = hi1 * cs1.x + lo1 * cs1.y;
      lo0 = a0; hi0 = b0; lo1 = a1; hi1 = b1;
    }
    const uint32_t lo = pack2_bf16(lo0, lo1), hi = pack2_bf16(hi0, hi1);
    if (head < n_q_heads) {
      const int kvh = head / group, r = (head % group) * window + (row - s * window);
      uint16_t* base = q + ((size_t)s * n_kv_heads + kvh) * r_pad * head_dim;
      *(uint32_t*)(base + pk_off(r, j0, head_dim)) = lo;
      *(uint32_t*)(base + pk_off(r, j0 + half, head_dim)) = hi;
      return;
    }
    const int blk = block_table[(size_t)s * max_blocks_per_seq + (pos >> 4)];
    const int tok = pos & 15;
    if (head < n_q_heads + n_kv_heads) {
      uint16_t* tile = k_plane + ((size_t)blk * n_kv_heads + (head - n_q_heads)) * 16 * head_dim;
      *(uint32_t*)(tile + ((j0 >> 3) * 16 + tok) * 8 + (j0 & 7)) = lo;
      *(uint32_t*)(tile + (((j0 + half) >> 3) * 16 + tok) * 8 + (j0 & 7)) = hi;
    } else {
      uint16_t* tile = v_plane + ((size_t)blk * n_kv_heads + (head - n_q_heads - n_kv_heads)) * 16 * head_dim;
      tile[j0 * 16 + tok] = (uint16_t)lo;
      tile[(j0 + 1) * 16 + tok] = (uint16_t)(lo >> 16);
      tile[(j0 + half) * 16 + tok] = (uint16_t)hi;
      tile[(j0 + half + 1) * 16 + tok] = (uint16_t)(hi >> 16);
    }
  }
};

struct ResidualEpi {
  float* resid;   // fp32 residual stream [m_pad][n], updated in place (one lane owns each element)
  int n;
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc) const {
    f32x4* p = (f32x4*)(resid + resid_off(row, nb * 16 + (lane >> 4) * 4, n));
    *p = *p + acc;
  }
};

__device__ inline float silu_f32(float z) { return z / (1.0f + __expf(-z)); }

struct SwigluEpi {
  uint16_t* hidden;  // tile layout [m_pad][ffn_k]
  int ffn_k;
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc) const {
    // acc[0], acc[1]: gate of hidden features f, f+1;  acc[2], acc[3]: up of the same features
    const int f = nb * 8 + (lane >> 4) * 2;
    const float h0 = silu_f32(acc[0]) * acc[2], h1 = silu_f32(acc[1]) * acc[3];
    *(uint32_t*)(hidden + pk_off(row, f, ffn_k)) = pack2_bf16(h0, h1);
  }
};

struct LogitsEpi {
  const int32_t* row_pos;
  const int32_t* row_seq;
  const int32_t* dump_slot;
  float* out_logits;   // [n_dump][window][vocab] or null
  float2* amax;        // [m_pad][n_blocks]
  int window, vocab, n_blocks;
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc) const {
    const int n0 = nb * 16 + (lane >> 4) * 4;
    if (out_logits && row_pos[row] >= 0) {
      const int s = row_seq[row], slot = dump_slot[s];
      if (slot >= 0)
        *(f32x4*)(out_logits + ((size_t)slot * window + (row - s * window)) * vocab + n0) = acc;
    }
    // best of this lane's 4 features (ascending index, strict '>' keeps the lowest on ties) ...
    float bv = acc[0];
    int bi = n0;
#pragma unroll
    for (int e = 1; e < 4; ++e)
      if (acc[e] > bv) { bv = acc[e]; bi = n0 + e; }
    // ... then of the 4 lanes that hold the token's other features of this block
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane < 16) amax[(size_t)row * n_blocks + nb] = make_float2(bv, __int_as_float(bi));
  }
};

// Streaming kernel: every wave owns one block of 16 features and MB blocks of 16
// tokens, reads its weight tiles once, straight from HBM into registers (1 KiB
// per load instruction, fully coalesced thanks to the tile layout), and its
// activation tiles through the caches.  4 waves per workgroup, no LDS, no barrier.
template <int MB, class Epi>
__global__ __launch_bounds__(256) void gemm_stream_kernel(const bf16x8* __restrict__ w, const bf16x8* __restrict__ x,
                                                          int n_blocks, int k_tiles, Epi epi) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nb = blockIdx.x * 4 + wave;
  if (nb >= n_blocks) return;
  const int mb0 = blockIdx.y * MB;
  const bf16x8* wp = w + (size_t)nb * k_tiles * 64 + lane;
  const bf16x8* xp = x + (size_t)mb0 * k_tiles * 64 + lane;
  f32x4 acc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b) acc[b] = (f32x4){0.f, 0.f, 0.f, 0.f};
  // U weight tiles are requested before the first of them is used; the MFMA order stays k ascending
  constexpr int U = 8;
  int kt = 0;
  for (; kt + U <= k_tiles; kt += U) {
    bf16x8 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(wp + (size_t)(kt + u) * 64);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int b = 0; b < MB; ++b) acc[b] = mfma16(a[u], xp[((size_t)b * k_tiles + kt + u) * 64], acc[b]);
  }
  for (; kt < k_tiles; ++kt) {
    const bf16x8 a = __builtin_nontemporal_load(wp + (size_t)kt * 64);
#pragma unroll
    for (int b = 0; b < MB; ++b) acc[b] = mfma16(a, xp[((size_t)b * k_tiles + kt) * 64], acc[b]);
  }
#pragma unroll
  for (int b = 0; b < MB; ++b) epi(nb, lane, (mb0 + b) * 16 + (lane & 15), acc[b]);
}

// Small-batch kernel (at most 64 tokens): HBM-bound weight streaming.
// One workgroup of 4 waves per block of 16 features.  All 4 waves fetch the
// block's weight tiles, CH k-tiles per round (CH KiB in flight per workgroup,
// each wave fetching every 4th tile), and park them in LDS; waves 0 .. MB-1 then
// each advance one 16-token block's accumulator through the round's tiles in
// ascending k order, with their own activation tiles prefetched in registers.
// The next round's weight loads are issued before the current round is consumed.
// Only the fetch is spread over the waves: the accumulation order per output
// element is the one stated at the top of this file.
template <int MB, class Epi>
__global__ __launch_bounds__(256) void gemm_coop_kernel(const bf16x8* __restrict__ w, const bf16x8* __restrict__ x,
                                                        int k_tiles, Epi epi) {
  constexpr int CH = 32;
  __shared__ bf16x8 wlds[CH * 64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nb = blockIdx.x;
  const bf16x8* wp = w + (size_t)nb * k_tiles * 64 + lane;
  const bf16x8* xp = x + (size_t)wave * k_tiles * 64 + lane;   // consumer `wave` owns token block `wave`
  const bool consumer = wave < MB;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  bf16x8 wr[CH / 4], xr[CH];
#pragma unroll
  for (int i = 0; i < CH / 4; ++i)
    if (i * 4 + wave < k_tiles) wr[i] = __builtin_nontemporal_load(wp + (size_t)(i * 4 + wave) * 64);
  if (consumer) {
#pragma unroll
    for (int j = 0; j < CH; ++j)
      if (j < k_tiles) xr[j] = xp[(size_t)j * 64];
  }
  for (int c0 = 0; c0 < k_tiles; c0 += CH) {
    const int nt = min(CH, k_tiles - c0);
#pragma unroll
    for (int i = 0; i < CH / 4; ++i)
      if (i * 4 + wave < nt) wlds[(i * 4 + wave) * 64 + lane] = wr[i];
    __syncthreads();
    const int n1 = c0 + CH;   // first tile of the next round
#pragma unroll
    for (int i = 0; i < CH / 4; ++i)
      if (n1 + i * 4 + wave < k_tiles) wr[i] = __builtin_nontemporal_load(wp + (size_t)(n1 + i * 4 + wave) * 64);
    if (consumer) {
#pragma unroll
      for (int j = 0; j < CH; ++j)
        if (j < nt) acc = mfma16(wlds[j * 64 + lane], xr[j], acc);
#pragma unroll
      for (int j = 0; j < CH; ++j)
        if (n1 + j < k_tiles) xr[j] = xp[(size_t)(n1 + j) * 64];
    }
    __syncthreads();
  }
  if (consumer) epi(nb, lane, wave * 16 + (lane & 15), acc);
}

template <class Epi>
void launch_stream(const uint16_t* w, const uint16_t* x, int n_blocks, int k_padded, int m_pad, const Epi& epi,
                   hipStream_t st) {
  const int k_tiles = k_padded / 32;
  const bf16x8* wp = (const bf16x8*)w;
  const bf16x8* xp = (const bf16x8*)x;
  if (m_pad == 16) {
    gemm_coop_kernel<1, Epi><<<n_blocks, 256, 0, st>>>(wp, xp, k_tiles, epi);
  } else if (m_pad == 32) {
    gemm_coop_kernel<2, Epi><<<n_blocks, 256, 0, st>>>(wp, xp, k_tiles, epi);
  } else if (m_pad == 64) {
    gemm_coop_kernel<4, Epi><<<n_blocks, 256, 0, st>>>(wp, xp, k_tiles, epi);
  } else {   // m_pad is a multiple of 64
    const unsigned gx = (unsigned)((n_blocks + 3) / 4);
    gemm_stream_kernel<4, Epi><<<dim3(gx, m_pad / 64), 256, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
  }
}

}  // namespace

void launch_gemm_qkv(const llm42_model* m, int layer, const llm42_kv_cache* kv, int window, const Workspace& ws,
                     hipStream_t st) {
  const llm42_config& c = m->cfg;
  const size_t plane = (size_t)kv->num_blocks * c.n_kv_heads * 16 * c.head_dim;
  QkvEpi e;
  e.rope = (const float2*)m->rope;
  e.row_pos = ws.row_pos;
  e.row_seq = ws.row_seq;
  e.block_table = kv->block_table;
  e.q = ws.q;
  e.k_plane = (uint16_t*)kv->kv_base + ((size_t)layer * 2 + 0) * plane;
  e.v_plane = (uint16_t*)kv->kv_base + ((size_t)layer * 2 + 1) * plane;
  e.n_q_heads = c.n_q_heads;
  e.n_kv_heads = c.n_kv_heads;
  e.head_dim = c.head_dim;
  e.group = m->group;
  e.window = window;
  e.r_pad = ws.r_pad;
  e.max_blocks_per_seq = kv->max_blocks_per_seq;
  launch_stream(m->layers[layer].wqkv, ws.normed, m->n_qkv / 16, c.d_model, ws.m_pad, e, st);
}

void launch_gemm_residual(const uint16_t* w, const uint16_t* x, float* resid, int n, int k_padded,
                          const Workspace& ws, hipStream_t st) {
  ResidualEpi e{resid, n};
  launch_stream(w, x, n / 16, k_padded, ws.m_pad, e, st);
}

void launch_gemm_swiglu(const llm42_model* m, int layer, const Workspace& ws, hipStream_t st) {
  SwigluEpi e{ws.hidden, m->ffn_k};
  launch_stream(m->layers[layer].wgu, ws.normed, m->gu_blocks, m->cfg.d_model, ws.m_pad, e, st);
}

void launch_gemm_logits(const llm42_model* m, int window, float* out_logits, const Workspace& ws, hipStream_t st) {
  LogitsEpi e;
  e.row_pos = ws.row_pos;
  e.row_seq = ws.row_seq;
  e.dump_slot = ws.dump_slot;
  e.out_logits = out_logits;
  e.amax = ws.amax;
  e.window = window;
  e.vocab = m->cfg.vocab;
  e.n_blocks = m->cfg.vocab / 16;
  launch_stream(m->lm_head, ws.normed, m->cfg.vocab / 16, m->cfg.d_model, ws.m_pad, e, st);
}
