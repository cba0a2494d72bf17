// Greedy sampler (merge of the per-block arg-max partials written by the LM-head
// GEMM) and the integer commit / rollback kernel.
#include "llm42_dev.h"

namespace {

__device__ inline void take_better(float& bv, int& bi, float ov, int oi) {
  if (ov > bv || (ov == bv && oi < bi)) {
    bv = ov;
    bi = oi;
  }
}

// One workgroup per row.  max with the lowest-index tie-break is associative and
// commutative, so the order of this reduction cannot change the result.
__global__ __launch_bounds__(256) void argmax_merge_kernel(const float2* __restrict__ amax,
                                                           const int32_t* __restrict__ row_pos, int n_blocks,
                                                           int32_t* __restrict__ out_tokens) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int row = blockIdx.x;
  if (row_pos[row] < 0) return;   // dead row: out_tokens stays -1 (whole workgroup leaves)
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  const float2* p = amax + (size_t)row * n_blocks;
  constexpr int U = 8;                                    // partials in flight per thread
  int b = threadIdx.x;
  for (; b + (U - 1) * 256 < n_blocks; b += U * 256) {
    float2 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = p[b + u * 256];
#pragma unroll
    for (int u = 0; u < U; ++u) take_better(bv, bi, v[u].x, __float_as_int(v[u].y));
  }
  for (; b < n_blocks; b += 256) {
    const float2 v = p[b];
    take_better(bv, bi, v.x, __float_as_int(v.y));
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) take_better(bv, bi, __shfl_xor(bv, off), __shfl_xor(bi, off));
  if ((threadIdx.x & 63) == 0) {
    sv[threadIdx.x >> 6] = bv;
    si[threadIdx.x >> 6] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) take_better(bv, bi, sv[w], si[w]);
    out_tokens[row] = bi;
  }
}

// One thread per sequence: count the leading candidates that the verifier
// reproduced, commit them plus the verifier's next token, truncate the length.
__global__ void commit_kernel(const int32_t* __restrict__ candidates, const int32_t* __restrict__ out_tokens,
                              const int32_t* __restrict__ n_valid, int num_seqs, int window, int32_t* seq_lens,
                              int32_t* committed_counts, int32_t* committed_tokens, int32_t* rolled_back_counts) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= num_seqs) return;
  const int32_t* x = candidates + (size_t)s * window;
  const int32_t* y = out_tokens + (size_t)s * window;
  int32_t* out = committed_tokens + (size_t)s * window;
  int n = n_valid ? n_valid[s] : window;
  n = min(max(n, 1), window);
  if (y[0] < 0) {   // skipped by the verifier: nothing to commit
    committed_counts[s] = 0;
    if (rolled_back_counts) rolled_back_counts[s] = 0;
    for (int i = 0; i < window; ++i) out[i] = -1;
    return;
  }
  int m = 0;
  while (m < n - 1 && x[m + 1] == y[m]) ++m;
  for (int i = 0; i < window; ++i) out[i] = i <= m ? y[i] : -1;
  committed_counts[s] = m + 1;
  if (rolled_back_counts) rolled_back_counts[s] = n - 1 - m;
  seq_lens[s] += m + 1;
}

}  // namespace

void launch_argmax_merge(const llm42_model* m, int num_seqs, int window, int32_t* out_tokens, const Workspace& ws,
                         hipStream_t st) {
  argmax_merge_kernel<<<num_seqs * window, 256, 0, st>>>(ws.amax, ws.row_pos, m->cfg.vocab / 16, out_tokens);
}

void launch_commit(const int32_t* candidates, const int32_t* out_tokens, const int32_t* n_valid, int num_seqs,
                   int window, int32_t* seq_lens, int32_t* committed_counts, int32_t* committed_tokens,
                   int32_t* rolled_back_counts, hipStream_t st) {
  commit_kernel<<<(num_seqs + 63) / 64, 64, 0, st>>>(candidates, out_tokens, n_valid, num_seqs, window, seq_lens,
                                                     committed_counts, committed_tokens, rolled_back_counts);
}
