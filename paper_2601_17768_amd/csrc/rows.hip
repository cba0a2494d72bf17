// Row-wise kernels of the verifier pass: input validation and row metadata,
// embedding gather, RMSNorm.
#include "llm42_dev.h"

namespace {

// One workgroup per sequence.  Validates what only the device can see (lengths,
// block-table entries, token ids) and writes the row metadata every later kernel
// uses.  A sequence that fails a check is switched off as a whole: its rows get
// position -1, no KV slot of it is read or written and its outputs are -1.
__global__ void prepare_kernel(const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ candidates,
                               const int32_t* __restrict__ n_valid, const int32_t* __restrict__ block_table,
                               int max_blocks_per_seq, int64_t num_blocks, int window, int max_context, int vocab,
                               const int32_t* __restrict__ dump_seq_ids, int n_dump, int32_t* out_tokens,
                               int32_t* seq_status, int32_t* row_pos, int32_t* row_seq, int32_t* ws_len,
                               int32_t* ws_n, int32_t* dump_slot, const float2* __restrict__ rope, int half_dim,
                               int32_t* row_blk, float2* row_rope, int min_n, int status_or,
                               uint16_t* __restrict__ attn_zero, int d_attn) {
  __shared__ int status;
  const int s = blockIdx.x;
  if (threadIdx.x == 0) status = 0;
  __syncthreads();
  const int L = seq_lens[s];
  const int n = n_valid ? n_valid[s] : window;
  int bad = 0;
  // (min_n is 1; a prefill pass passes 0: a sequence whose prompt has ended takes no part in the pass)
  if (L < 0 || n < min_n || n > window || (int64_t)L + n > max_context) bad = LLM42_SEQ_BAD_LENGTH;
  if (!bad) {
    const int blocks = (L + n + LLM42_KV_BLOCK - 1) / LLM42_KV_BLOCK;   // <= max_blocks_per_seq (host checked)
    for (int b = threadIdx.x; b < blocks; b += blockDim.x) {
      const int id = block_table[(size_t)s * max_blocks_per_seq + b];
      if (id < 0 || id >= num_blocks) bad |= LLM42_SEQ_BAD_BLOCK;
    }
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      const int t = candidates[(size_t)s * window + i];
      if (t < 0 || t >= vocab) bad |= LLM42_SEQ_BAD_TOKEN;
    }
  }
  if (bad) atomicOr(&status, bad);   // integer OR: order-free
  __syncthreads();
  const int st = status;
  for (int i = threadIdx.x; i < window; i += blockDim.x) {
    const int row = s * window + i;
    const bool live = st == 0 && i < n;
    row_pos[row] = live ? L + i : -1;
    row_seq[row] = s;
    // where the row's K and V go (a block id that passed the check above), for the QKV epilogue
    row_blk[row] = live ? block_table[(size_t)s * max_blocks_per_seq + ((L + i) >> 4)] : 0;
    out_tokens[row] = -1;              // overwritten by the arg-max merge for live rows
  }
  // the rotary factors of every live row, laid out by row so that the QKV epilogue finds them without
  // knowing the position first
  if (st == 0) {
    for (int e = threadIdx.x; e < n * half_dim; e += blockDim.x) {
      const int i = e / half_dim, j = e - i * half_dim;
      row_rope[(size_t)(s * window + i) * half_dim + j] = rope[(size_t)(L + i) * half_dim + j];
    }
  }
  // Without a merge pass (attn_zero given) nothing writes the attention output of rows that take no part:
  // give them zeros once, so that everything downstream of them stays finite.
  if (attn_zero) {
    const int chunks = d_attn / 8;
    for (int e = threadIdx.x; e < window * chunks; e += blockDim.x) {
      const int i = e / chunks, c8 = e - i * chunks;
      if (st != 0 || i >= n) *(uint4*)(attn_zero + pk_off(s * window + i, c8 * 8, d_attn)) = make_uint4(0, 0, 0, 0);
    }
  }
  if (threadIdx.x == 0) {
    ws_len[s] = st == 0 && n > 0 ? L : -1;
    ws_n[s] = st == 0 ? n : 0;
    if (seq_status) seq_status[s] = status_or ? (seq_status[s] | st) : st;
    int slot = -1;
    for (int j = 0; j < n_dump; ++j)
      if (dump_seq_ids[j] == s) slot = j;
    dump_slot[s] = slot;
  }
}

// Rows beyond num_seqs*window that only pad the GEMM grid.
__global__ void prepare_pad_rows_kernel(int32_t* row_pos, int32_t* row_seq, int32_t* row_blk, int from, int to) {
  const int r = from + blockIdx.x * blockDim.x + threadIdx.x;
  if (r < to) {
    row_pos[r] = -1;
    row_seq[r] = 0;
    row_blk[r] = 0;
  }
}

// Prefill, pass `chunk_index`: cuts the next `window` prompt tokens of every sequence into the
// candidate rows of one verifier pass.  One workgroup per sequence.
__global__ void prefill_window_kernel(const int32_t* __restrict__ prompt_tokens, const int32_t* __restrict__ prompt_offsets,
                                      const int32_t* __restrict__ seq_lens, int window, int chunk_index,
                                      int max_prompt_len, int32_t* __restrict__ cand, int32_t* __restrict__ n_valid,
                                      int32_t* __restrict__ lens_now, int32_t* __restrict__ seq_status,
                                      int32_t* __restrict__ out_next) {
  const int s = blockIdx.x;
  const int off = prompt_offsets[s], len = prompt_offsets[s + 1] - off;
  const int start = chunk_index * window;
  const bool bad = off < 0 || len < 0 || len > max_prompt_len;
  const int n = bad ? 0 : min(max(len - start, 0), window);
  for (int i = threadIdx.x; i < window; i += blockDim.x) cand[(size_t)s * window + i] = i < n ? prompt_tokens[off + start + i] : 0;
  if (threadIdx.x == 0) {
    n_valid[s] = n;
    lens_now[s] = seq_lens[s] + (n > 0 ? start : 0);
    if (chunk_index == 0) {
      if (seq_status) seq_status[s] = bad ? LLM42_SEQ_BAD_LENGTH : 0;
      out_next[s] = -1;
    }
  }
}

// After a prefill pass: the sequences whose last prompt token was in this pass take the pass's
// token for that row.  A sequence that failed a check keeps -1.
__global__ void prefill_pick_kernel(const int32_t* __restrict__ prompt_offsets, int window, int chunk_index,
                                    const int32_t* __restrict__ pass_tokens, int num_seqs,
                                    const int32_t* __restrict__ seq_status, int32_t* __restrict__ out_next) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= num_seqs) return;
  const int len = prompt_offsets[s + 1] - prompt_offsets[s];
  const int last = len - 1 - chunk_index * window;        // row of the last prompt token in this pass
  if (len > 0 && last >= 0 && last < window)
    out_next[s] = seq_status[s] == 0 ? pass_tokens[(size_t)s * window + last] : -1;
}

// One wave per 16 rows x 32 features of the residual stream: lane
// (row = lane % 16, g = lane / 16) converts 8 features of its row's embedding to
// fp32 (exact).  Dead rows get zeros so that everything downstream stays finite.
__global__ void embed_kernel(const uint16_t* __restrict__ table, const int32_t* __restrict__ candidates,
                             const int32_t* __restrict__ row_pos, int m_rows, int d, float* __restrict__ resid) {
  const int col_tiles = d / 32;
  const size_t tile = (size_t)blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  const int lane = threadIdx.x & 63;
  const int rb = (int)(tile / col_tiles), cb = (int)(tile % col_tiles);
  const int row = rb * 16 + (lane & 15);
  const int feat = cb * 32 + (lane >> 4) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < m_rows && row_pos[row] >= 0) {
    const int tok = candidates[row];
    v = *(const uint4*)(table + (size_t)tok * d + feat);
  }
  f32x4 lo = {bf16_bits_to_f32(v.x & 0xFFFFu), bf16_bits_to_f32(v.x >> 16), bf16_bits_to_f32(v.y & 0xFFFFu),
              bf16_bits_to_f32(v.y >> 16)};
  f32x4 hi = {bf16_bits_to_f32(v.z & 0xFFFFu), bf16_bits_to_f32(v.z >> 16), bf16_bits_to_f32(v.w & 0xFFFFu),
              bf16_bits_to_f32(v.w >> 16)};
  *(f32x4*)(resid + resid_off(row, feat, d)) = lo;
  *(f32x4*)(resid + resid_off(row, feat + 4, d)) = hi;
}

// Sum of the 64 per-lane partial sums of squares of a row (lane w*4+g owns p[w][g]) in the fixed
// order stated at rmsnorm_kernel, and the row's 1 / sqrt(mean square + eps).
__device__ inline float row_inv_rms(float ss, int d, float eps) {
  ss += __shfl_xor(ss, 1);
  ss += __shfl_xor(ss, 2);
  float total = __shfl(ss, 0);
#pragma unroll
  for (int ww = 1; ww < 16; ++ww) total += __shfl(ss, ww * 4);
  return 1.0f / __builtin_sqrtf(total / (float)d + eps);
}

// y[f .. f+7] = bf16(x * inv * gain), written into the tile layout; yr points at the row's feature 0.
__device__ inline void emit_normed(uint4* yr, int f, const f32x4 a, const f32x4 b, const uint4 gv, float inv) {
  uint4 o;
  o.x = pack2_bf16(a[0] * inv * bf16_bits_to_f32(gv.x & 0xFFFFu), a[1] * inv * bf16_bits_to_f32(gv.x >> 16));
  o.y = pack2_bf16(a[2] * inv * bf16_bits_to_f32(gv.y & 0xFFFFu), a[3] * inv * bf16_bits_to_f32(gv.y >> 16));
  o.z = pack2_bf16(b[0] * inv * bf16_bits_to_f32(gv.z & 0xFFFFu), b[1] * inv * bf16_bits_to_f32(gv.z >> 16));
  o.w = pack2_bf16(b[2] * inv * bf16_bits_to_f32(gv.w & 0xFFFFu), b[3] * inv * bf16_bits_to_f32(gv.w >> 16));
  yr[(f >> 5) * 64 + ((f & 31) >> 3) * 16] = o;
}

// RMSNorm, one wave per row (1 or 4 rows per workgroup); fp32 residual stream in, bf16
// tile layout (the next GEMM's activation operand) out.
// Reduction schedule per row (a function of d only): 64 partial sums p[w][g],
// w = 0..15, g = 0..3; p[w][g] accumulates, in ascending feature order, the squares
// of features t*32 + g*8 .. +7 for t = w, w+16, w+32, ...; then per w the four g
// are added as (p[w][g] + p[w][g^1]) + (p[w][g^2] + p[w][g^3]), and the 16 results
// are added in ascending w.  Lane w*4+g of the row's wave owns p[w][g].
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const uint16_t* __restrict__ gain,
                                                      uint16_t* __restrict__ y, int m_pad, int d, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= m_pad) return;
  const int w = lane >> 2, g = lane & 3;
  const int col_tiles = d / 32;
  constexpr int U = 8;                                   // tiles in flight per lane
  const int full = col_tiles / (16 * U);                 // rounds in which every lane has U tiles
  const float* xr = x + resid_off(row, 0, d);            // feature f of this row: xr + (f / 4) * 64 + f % 4
  uint4* yr = (uint4*)(y + pk_off(row, 0, d));           // 8 features from f (f % 8 == 0): yr + (f/32)*64 + ((f%32)/8)*16
  float ss = 0.f;
  // (no load sits behind a per-load condition: the compiler would serialise such loads)
  if (full == 1 && col_tiles == 16 * U) {
    // d = 4096: the lane's whole share of the row (and of the gains) stays in registers
    f32x4 a[U], b[U];
    uint4 gv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int f = (u * 16 + w) * 32 + g * 8;
      a[u] = *(const f32x4*)(xr + (f >> 2) * 64);
      b[u] = *(const f32x4*)(xr + (f >> 2) * 64 + 64);
      gv[u] = *(const uint4*)(gain + f);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(a[u][i], a[u][i], ss);
#pragma unroll
      for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(b[u][i], b[u][i], ss);
    }
    const float inv = row_inv_rms(ss, d, eps);
#pragma unroll
    for (int u = 0; u < U; ++u) emit_normed(yr, (u * 16 + w) * 32 + g * 8, a[u], b[u], gv[u], inv);
    return;
  }
  for (int rd = 0; rd < full; ++rd) {
    f32x4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int f = ((rd * U + u) * 16 + w) * 32 + g * 8;
      a[u] = *(const f32x4*)(xr + (f >> 2) * 64);
      b[u] = *(const f32x4*)(xr + (f >> 2) * 64 + 64);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(a[u][i], a[u][i], ss);
#pragma unroll
      for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(b[u][i], b[u][i], ss);
    }
  }
  for (int t = full * U * 16 + w; t < col_tiles; t += 16) {
    const int f = t * 32 + g * 8;
    const f32x4 a = *(const f32x4*)(xr + (f >> 2) * 64), b = *(const f32x4*)(xr + (f >> 2) * 64 + 64);
#pragma unroll
    for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(a[i], a[i], ss);
#pragma unroll
    for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(b[i], b[i], ss);
  }
  const float inv = row_inv_rms(ss, d, eps);
  for (int rd = 0; rd < full; ++rd) {
    f32x4 a[U], b[U];
    uint4 gv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int f = ((rd * U + u) * 16 + w) * 32 + g * 8;
      a[u] = *(const f32x4*)(xr + (f >> 2) * 64);
      b[u] = *(const f32x4*)(xr + (f >> 2) * 64 + 64);
      gv[u] = *(const uint4*)(gain + f);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) emit_normed(yr, ((rd * U + u) * 16 + w) * 32 + g * 8, a[u], b[u], gv[u], inv);
  }
  for (int t = full * U * 16 + w; t < col_tiles; t += 16) {
    const int f = t * 32 + g * 8;
    emit_normed(yr, f, *(const f32x4*)(xr + (f >> 2) * 64), *(const f32x4*)(xr + (f >> 2) * 64 + 64),
                *(const uint4*)(gain + f), inv);
  }
}

// RMSNorm for many rows at d = 4096: one workgroup of 1024 threads per block of 16 rows, thread
// (w, g, r) owning the partial sum p[w][g] of row r - the same 64 partials per row, accumulated in
// the same order and combined in the same tree as in rmsnorm_kernel, so the bits are the same; only
// the work distribution differs.  With 16 rows of a token block side by side every 16-byte piece of
// the residual stream and of the output tiles is read or written as part of a full 256-byte run
// (the wave-per-row kernel touches every 128-byte line for half of its bytes).
__global__ __launch_bounds__(1024) void rmsnorm_block_kernel(const float* __restrict__ x,
                                                             const uint16_t* __restrict__ gain,
                                                             uint16_t* __restrict__ y, float eps) {
  constexpr int D = 4096, U = 8;                         // tiles of 32 features per thread: t = u * 16 + w
  __shared__ float part[64][16];
  __shared__ float inv_s[16];
  const int r = threadIdx.x & 15, wg = threadIdx.x >> 4, w = wg >> 2, g = wg & 3;
  const int row = blockIdx.x * 16 + r;
  const float* xr = x + resid_off(row, 0, D);
  uint4* yr = (uint4*)(y + pk_off(row, 0, D));
  f32x4 a[U], b[U];
  uint4 gv[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int f = (u * 16 + w) * 32 + g * 8;
    a[u] = *(const f32x4*)(xr + (f >> 2) * 64);
    b[u] = *(const f32x4*)(xr + (f >> 2) * 64 + 64);
    gv[u] = *(const uint4*)(gain + f);
  }
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(a[u][i], a[u][i], ss);
#pragma unroll
    for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(b[u][i], b[u][i], ss);
  }
  part[wg][r] = ss;
  __syncthreads();
  if (threadIdx.x < 16) {
    float total = 0.f;
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) {
      const float s4 = (part[ww * 4][r] + part[ww * 4 + 1][r]) + (part[ww * 4 + 2][r] + part[ww * 4 + 3][r]);
      total = ww == 0 ? s4 : total + s4;
    }
    inv_s[r] = 1.0f / __builtin_sqrtf(total / (float)D + eps);
  }
  __syncthreads();
  const float inv = inv_s[r];
#pragma unroll
  for (int u = 0; u < U; ++u) emit_normed(yr, (u * 16 + w) * 32 + g * 8, a[u], b[u], gv[u], inv);
}

}  // namespace

void launch_prepare(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                    const int32_t* candidates, const int32_t* n_valid, int num_seqs, int window,
                    int max_context, const int32_t* dump_seq_ids, int n_dump, int32_t* out_tokens,
                    int32_t* seq_status, const Workspace& ws, hipStream_t st, bool prefill_pass) {
  prepare_kernel<<<num_seqs, 256, 0, st>>>(seq_lens, candidates, n_valid, kv->block_table, kv->max_blocks_per_seq,
                                          kv->num_blocks, window, max_context, m->cfg.vocab, dump_seq_ids, n_dump,
                                          out_tokens, seq_status, ws.row_pos, ws.row_seq, ws.seq_len, ws.seq_n,
                                          ws.dump_slot, (const float2*)m->rope, m->cfg.head_dim / 2, ws.row_blk,
                                          ws.row_rope, prefill_pass ? 0 : 1, prefill_pass ? 1 : 0,
                                          ws.attn_direct || ws.attn_seq ? ws.attn : nullptr, m->d_attn);
  if (ws.m_pad > ws.m_rows)
    prepare_pad_rows_kernel<<<(ws.m_pad - ws.m_rows + 63) / 64, 64, 0, st>>>(ws.row_pos, ws.row_seq, ws.row_blk,
                                                                            ws.m_rows, ws.m_pad);
}

void launch_prefill_window(const int32_t* prompt_tokens, const int32_t* prompt_offsets, const int32_t* seq_lens,
                           int num_seqs, int window, int chunk_index, int max_prompt_len, int32_t* cand,
                           int32_t* n_valid, int32_t* lens_now, int32_t* seq_status, int32_t* out_next, hipStream_t st) {
  prefill_window_kernel<<<num_seqs, 64, 0, st>>>(prompt_tokens, prompt_offsets, seq_lens, window, chunk_index, max_prompt_len, cand,
                                                 n_valid, lens_now, seq_status, out_next);
}

void launch_prefill_pick(const int32_t* prompt_offsets, int num_seqs, int window, int chunk_index,
                         const int32_t* pass_tokens, const int32_t* seq_status, int32_t* out_next, hipStream_t st) {
  prefill_pick_kernel<<<(num_seqs + 255) / 256, 256, 0, st>>>(prompt_offsets, window, chunk_index, pass_tokens, num_seqs,
                                                             seq_status, out_next);
}

void launch_embed(const llm42_model* m, const int32_t* candidates, const Workspace& ws, hipStream_t st) {
  const int tiles = ws.m_pad / 16 * (m->cfg.d_model / 32);   // a multiple of 4 (d_model % 128 == 0 is checked)
  embed_kernel<<<tiles / 4, 256, 0, st>>>(m->embed, candidates, ws.row_pos, ws.m_rows, m->cfg.d_model, ws.resid);
}

void launch_rmsnorm(const float* x, const uint16_t* gain, uint16_t* y, int m_pad, int d, float eps,
                    hipStream_t st) {
  if (d == 4096 && m_pad >= 256 && m_pad % 16 == 0) rmsnorm_block_kernel<<<m_pad / 16, 1024, 0, st>>>(x, gain, y, eps);
  // few rows: one wave per workgroup, so that the rows' loads are spread over as many CUs as there are rows
  // (measured at 512 .. 1024 rows as well: there the block kernel is up to twice as fast)
  else if (m_pad <= 256) rmsnorm_kernel<<<m_pad, 64, 0, st>>>(x, gain, y, m_pad, d, eps);
  else rmsnorm_kernel<<<(m_pad + 3) / 4, 256, 0, st>>>(x, gain, y, m_pad, d, eps);
}
