// Weight repacking: plain row-major bf16 [out][in] matrices -> tile layout
// (see llm42_dev.h).  Runs once, inside llm42_model_create.
//
// Every kernel here assigns one thread to one 16-byte group of the destination
// (8 consecutive input features of one packed row) and copies it from the
// source row that the packing maps there, or writes zeros for padding.
#include "llm42_dev.h"

namespace {

// Decompose a destination group index into (packed row, first column).
__device__ inline void group_to_rc(size_t grp, int col_tiles, int& row, int& col) {
  const int within = (int)(grp & 63);          // group inside the 1 KiB tile
  const size_t tile = grp >> 6;
  const int cb = (int)(tile % col_tiles);
  const int rb = (int)(tile / col_tiles);
  row = rb * 16 + (within & 15);
  col = cb * 32 + (within >> 4) * 8;
}

__global__ void pack_plain_kernel(const uint16_t* __restrict__ src, uint4* __restrict__ dst, int rows, int cols,
                                  int col_tiles, size_t groups) {
  const size_t grp = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (grp >= groups) return;
  int r, c;
  group_to_rc(grp, col_tiles, r, c);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (r < rows && c < cols) v = *(const uint4*)(src + (size_t)r * cols + c);   // cols % 8 == 0
  dst[grp] = v;
}

// Packed row n of the fused QKV matrix: head = n / head_dim over the
// concatenation [q heads | k heads | v heads]; inside a head the packed index
// pn = n % head_dim maps to feature
//     j0 + (e & 1) + (e >= 2 ? head_dim / 2 : 0),  j0 = (pn / 16) * 8 + ((pn % 16) / 4) * 2,  e = pn % 4,
// so that the four consecutive packed rows a lane of the result tile owns are
// two rotary pairs (j, j + head_dim/2), (j+1, j+1 + head_dim/2).
__global__ void pack_qkv_kernel(const uint16_t* __restrict__ wq, const uint16_t* __restrict__ wk,
                                const uint16_t* __restrict__ wv, uint4* __restrict__ dst, int n_q_heads,
                                int n_kv_heads, int head_dim, int d_model, size_t groups) {
  const size_t grp = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (grp >= groups) return;
  int n, c;
  group_to_rc(grp, d_model / 32, n, c);
  const int head = n / head_dim, pn = n % head_dim, e = pn & 3;
  const int j0 = (pn >> 4) * 8 + ((pn & 15) >> 2) * 2;
  const int feat = j0 + (e & 1) + (e >= 2 ? head_dim / 2 : 0);
  const uint16_t* src;
  int h = head;
  if (h < n_q_heads) {
    src = wq;
  } else if (h < n_q_heads + n_kv_heads) {
    src = wk;
    h -= n_q_heads;
  } else {
    src = wv;
    h -= n_q_heads + n_kv_heads;
  }
  dst[grp] = *(const uint4*)(src + ((size_t)h * head_dim + feat) * d_model + c);
}

// Packed row n of the fused gate/up matrix: hidden feature 8*(n/16) + 2*((n%16)/4) + (n & 1),
// taken from the gate matrix when (n % 4) < 2 and from the up matrix otherwise, so
// a lane of the result tile owns gate and up of two neighbouring hidden features.
// Hidden features >= d_ffn (padding up to the down projection's padded K) are zero rows.
__global__ void pack_gate_up_kernel(const uint16_t* __restrict__ wg, const uint16_t* __restrict__ wu,
                                    uint4* __restrict__ dst, int d_ffn, int d_model, size_t groups) {
  const size_t grp = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (grp >= groups) return;
  int n, c;
  group_to_rc(grp, d_model / 32, n, c);
  const int e = n & 3;
  const int feat = (n >> 4) * 8 + ((n & 15) >> 2) * 2 + (e & 1);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (feat < d_ffn) v = *(const uint4*)((e < 2 ? wg : wu) + (size_t)feat * d_model + c);
  dst[grp] = v;
}

inline unsigned blocks_for(size_t groups) { return (unsigned)((groups + 255) / 256); }

}  // namespace

void launch_pack_plain(const uint16_t* src, uint16_t* dst, int rows, int cols, int cols_padded, hipStream_t st) {
  const int rows_padded = (rows + 15) / 16 * 16;
  const size_t groups = (size_t)rows_padded * cols_padded / 8;
  pack_plain_kernel<<<blocks_for(groups), 256, 0, st>>>(src, (uint4*)dst, rows, cols, cols_padded / 32, groups);
}

void launch_pack_qkv(const uint16_t* wq, const uint16_t* wk, const uint16_t* wv, uint16_t* dst,
                     const llm42_config& c, hipStream_t st) {
  const size_t rows = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  const size_t groups = rows * c.d_model / 8;
  pack_qkv_kernel<<<blocks_for(groups), 256, 0, st>>>(wq, wk, wv, (uint4*)dst, c.n_q_heads, c.n_kv_heads,
                                                      c.head_dim, c.d_model, groups);
}

void launch_pack_gate_up(const uint16_t* wg, const uint16_t* wu, uint16_t* dst, int d_ffn, int gu_blocks,
                         int d_model, hipStream_t st) {
  const size_t groups = (size_t)gu_blocks * 16 * d_model / 8;
  pack_gate_up_kernel<<<blocks_for(groups), 256, 0, st>>>(wg, wu, (uint4*)dst, d_ffn, d_model, groups);
}
