// Device-side helpers and the launcher interface between the translation units
// of the verifier library (gfx950 only).
//
// Packed operand layout ("tile layout") used for every GEMM operand in HBM:
// a matrix [R][C] (R padded to 16, C padded to 32) is cut into tiles of
// 16 rows x 32 columns (1 KiB of bf16).  Tiles are stored row-block major
// (all column tiles of a 16-row block are contiguous) and inside a tile element
// (r, c) sits at ((c / 8) * 16 + r) * 8 + c % 8.  A tile is exactly one operand
// of v_mfma_f32_16x16x32_bf16 in lane order (lane = (c / 8) * 16 + r holds the
// 8 consecutive columns c & ~7 .. ), so a wave fetches an operand with one
// fully coalesced 16-byte-per-lane load and no shuffling.
//
// GEMMs are computed transposed, D[feature][token] = sum_k W[feature][k] X[token][k]:
// weights are the A operand, activations the B operand.  In the result tile a
// lane (token = lane % 16, g = lane / 16) holds features g*4 .. g*4+3 of its
// token, i.e. four consecutive features, which it can store straight back into
// the tile layout of the next GEMM's activation operand.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/llm42.h"
#include "../../include/llm42_measure.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;


__host__ __device__ inline size_t pk_off(int r, int c, int c_padded) {
  return ((size_t)(r >> 4) * (size_t)(c_padded >> 5) + (size_t)(c >> 5)) * 512 +
         (size_t)((((c & 31) >> 3) * 16 + (r & 15)) * 8 + (c & 7));
}

// Residual stream: fp32, [token block of 16][feature group of 4][token][4], so the four
// consecutive features a lane owns after a GEMM are one 16-byte access and a wave's
// accesses are contiguous.
__host__ __device__ inline size_t resid_off(int row, int feat, int n) {
  return (((size_t)(row >> 4) * (size_t)(n >> 2) + (size_t)(feat >> 2)) * 16 + (size_t)(row & 15)) * 4 + (feat & 3);
}

__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even on the bit pattern (inputs are finite here)
__device__ inline uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
// the same rounding for two values at once, by the hardware conversion (one instruction on gfx950)
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ inline uint32_t pack2_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// V tile of the KV cache: [feature block of 16][token group of 4][feature][4 tokens], the order in
// which the lanes of a P V operand read it (8 contiguous bytes per lane, 512 per wave).
__host__ __device__ inline int v_tile_off(int f, int t) {
  return (((f >> 4) * 4 + (t >> 2)) * 16 + (f & 15)) * 4 + (t & 3);
}

__device__ inline f32x4 mfma16(const bf16x8 a, const bf16x8 b, const f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// model and per-call plan (host side)
// ---------------------------------------------------------------------------
struct llm42_model {
  llm42_config cfg;
  int device;       // HIP device the model lives on
  int num_cus;      // compute units of that device
  int group;        // q heads per kv head
  int n_qkv;        // (n_q_heads + 2 n_kv_heads) * head_dim
  int d_attn;       // n_q_heads * head_dim
  int ffn_k;        // d_ffn padded to 32: K of the down projection
  int gu_blocks;    // packed gate/up feature blocks (16 packed rows = 8 hidden features)
  uint16_t* arena;  // one device allocation holding everything below
  size_t arena_bytes;
  uint16_t* embed;  // [vocab][d] row-major (gathered, never multiplied)
  uint16_t* final_norm;
  uint16_t* lm_head;  // packed [vocab][d]
  struct Layer {
    uint16_t *attn_norm, *wqkv, *wo, *ffn_norm, *wgu, *wdown;
  }* layers;          // host array
  float* rope;        // [max_position][head_dim/2][2] (cos, sin), fp32
};

// Workspace carving, identical in llm42_workspace_bytes and llm42_verify_window.
struct Workspace {
  int num_cus;    // compute units of the device
  int m_rows;     // num_seqs * window
  int m_pad;      // rows padded for the GEMM grid
  int r_pad;      // query rows per (seq, kv head) padded to 16
  int attn_units; // attention partial slots per row (chunks or supers, see attention.hip)
  bool attn_super; // one workgroup per super (many sequences) instead of per chunk
  bool attn_direct; // every sequence fits one super: the attention kernel writes the final output, no merge pass
  bool attn_seq;    // the call may take whole sequences as attention items (the plan kernel decides from the lengths)
  bool batch_chosen; // off the fixed schedule (fast-path decode step, cost-of-determinism measurement): the batch may
                     // choose the split of the residual projections and the attention partials
  int32_t *row_pos, *row_seq, *seq_len, *seq_n, *dump_slot;
  int32_t* row_blk;    // physical KV block that holds the row's position (0 for dead rows)
  float2* row_rope;    // [m_pad][head_dim/2] (cos, sin) at the row's position
  float* resid;
  uint16_t *normed, *q, *attn, *hidden;
  float *part_acc, *part_ml;
  int4* attn_items;     // (sequence, unit, length, rows) of every unit that holds keys, built once per call
  int32_t* attn_ctrl;   // [0] number of items, [1 + layer] work queue counter of that layer's attention launch,
                        // [1 + n_layers] 1 if the items are whole sequences
  size_t attn_ctrl_offset;   // byte offset of attn_ctrl in the workspace
  float* split_part;   // fp32 partials of a split GEMM on the large-batch path, [2][m_pad][d_model]
  float2* amax;   // [m_pad][vocab/16] (value, index bits)
  size_t bytes;
};

// ---------------------------------------------------------------------------
// launchers (each defined in the .hip file that holds its kernel)
// ---------------------------------------------------------------------------
void launch_pack_plain(const uint16_t* src, uint16_t* dst, int rows, int cols, int cols_padded, hipStream_t st);
void launch_pack_qkv(const uint16_t* wq, const uint16_t* wk, const uint16_t* wv, uint16_t* dst,
                     const llm42_config& c, hipStream_t st);
void launch_pack_gate_up(const uint16_t* wg, const uint16_t* wu, uint16_t* dst, int d_ffn, int gu_blocks,
                         int d_model, hipStream_t st);

void launch_prepare(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                    const int32_t* candidates, const int32_t* n_valid, int num_seqs, int window,
                    int max_context, const int32_t* dump_seq_ids, int n_dump, int32_t* out_tokens,
                    int32_t* seq_status, const Workspace& ws, hipStream_t st, bool prefill_pass);
void launch_prefill_window(const int32_t* prompt_tokens, const int32_t* prompt_offsets, const int32_t* seq_lens,
                           int num_seqs, int window, int chunk_index, int max_prompt_len, int32_t* cand,
                           int32_t* n_valid, int32_t* lens_now, int32_t* seq_status, int32_t* out_next, hipStream_t st);
void launch_prefill_pick(const int32_t* prompt_offsets, int num_seqs, int window, int chunk_index,
                         const int32_t* pass_tokens, const int32_t* seq_status, int32_t* out_next, hipStream_t st);
void launch_embed(const llm42_model* m, const int32_t* candidates, const Workspace& ws, hipStream_t st);
void launch_rmsnorm(const float* x, const uint16_t* gain, uint16_t* y, int m_pad, int d, float eps,
                    hipStream_t st);

void launch_gemm_qkv(const llm42_model* m, int layer, const llm42_kv_cache* kv, int window, const Workspace& ws,
                     hipStream_t st);
void launch_gemm_residual(const uint16_t* w, const uint16_t* x, float* resid, int n, int k_padded,
                          const Workspace& ws, hipStream_t st);
void launch_gemm_swiglu(const llm42_model* m, int layer, const Workspace& ws, hipStream_t st);
void launch_gemm_logits(const llm42_model* m, int window, float* out_logits, const llm42_sampling* sampling,
                        const Workspace& ws, hipStream_t st);

int attention_units(bool super_mode, int max_context);
void launch_attention_plan(const llm42_model* m, int num_seqs, int max_context, const Workspace& ws, hipStream_t st);
void launch_attention(const llm42_model* m, int layer, const llm42_kv_cache* kv, int num_seqs, int window,
                      int max_context, const Workspace& ws, hipStream_t st);
void launch_argmax_merge(const llm42_model* m, int num_seqs, int window, int32_t* out_tokens, const Workspace& ws,
                         hipStream_t st);
void launch_commit(const int32_t* candidates, const int32_t* out_tokens, const int32_t* n_valid, int num_seqs,
                   int window, int32_t* seq_lens, int32_t* committed_counts, int32_t* committed_tokens,
                   int32_t* rolled_back_counts, hipStream_t st);
