// bf16 MFMA GEMMs of the verifier pass, D[feature][token] = sum_k W[feature][k] X[token][k],
// with the layer-specific epilogues fused (rotary embedding + KV-cache write,
// residual add, SwiGLU, logits + arg-max partials).
//
// Reduction schedule (what fixes the bits of every output element): one fp32
// accumulator per element, started at zero, updated by v_mfma_f32_16x16x32_bf16
// over k-tiles 0, 1, 2, ... in ascending order; the two residual projections use two such
// accumulators, one per half of K, added once at the end (kSplit below), the other GEMMs one.  The
// schedule depends on K and on the kind of GEMM only.  How many token blocks a wave owns, how many waves share a
// workgroup and how the grid is shaped are work-distribution choices that do not
// touch it, so they may change with the number of rows.
#include <type_traits>

#include "llm42_dev.h"

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct QkvEpi {
  const float4* __restrict__ row_rope;    // [row][head_dim/4]: (cos, sin) of two consecutive rotary pairs at the row's position
  const int32_t* __restrict__ row_pos;
  const int32_t* __restrict__ row_seq;
  const int32_t* __restrict__ row_blk;    // physical KV block of the row's position
  uint16_t* q;               // [seq][kv head][r_pad][head_dim] tile layout, r = q-head-in-group * window + i
  uint16_t* k_plane;         // this layer's K tiles [block][kv head][16*head_dim]
  uint16_t* v_plane;
  int n_q_heads, n_kv_heads, head_dim, group, window, r_pad;

  // What the epilogue needs from memory besides the accumulators; requested when the kernel
  // starts so that its latency hides behind the weight stream.  Everything is indexed by the row
  // alone (the per-row block id and rotary factors are laid out once per call), so none of these
  // loads waits for another.
  struct Row {   // per token row
    int pos, s, blk;
  };
  struct Pre {   // per (token row, feature block)
    int pos, s, blk;
    float2 cs0, cs1;
  };
  __device__ Row row_info(int row) const {
    Row r;
    r.pos = row_pos[row];
    r.s = row_seq[row];
    r.blk = row_blk[row];
    return r;
  }
  __device__ Pre pre(int nb, int lane, int row, const Row& r) const {
    Pre p;
    p.pos = r.pos;
    p.s = r.s;
    p.blk = r.blk;
    const int j0 = (nb % (head_dim >> 4)) * 8 + (lane >> 4) * 2;
    const float4 cs = row_rope[(size_t)row * (head_dim >> 2) + (j0 >> 1)];
    p.cs0 = make_float2(cs.x, cs.y);
    p.cs1 = make_float2(cs.z, cs.w);
    return p;
  }
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc, const Pre& p) const {
    const int pos = p.pos;
    if (pos < 0) return;
    const int blocks_per_head = head_dim >> 4;
    const int head = nb / blocks_per_head, t = nb % blocks_per_head, g = lane >> 4;
    const int j0 = t * 8 + g * 2;           // features j0, j0+1 and their rotary partners j0 + hd/2, j0+1 + hd/2
    const int half = head_dim >> 1;
    const int s = p.s;
    float lo0 = acc[0], lo1 = acc[1], hi0 = acc[2], hi1 = acc[3];
    if (head < n_q_heads + n_kv_heads) {
      const float2 cs0 = p.cs0, cs1 = p.cs1;
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
    const int blk = p.blk;
    const int tok = pos & 15;
    if (head < n_q_heads + n_kv_heads) {
      uint16_t* tile = k_plane + ((size_t)blk * n_kv_heads + (head - n_q_heads)) * 16 * head_dim;
      *(uint32_t*)(tile + ((j0 >> 3) * 16 + tok) * 8 + (j0 & 7)) = lo;
      *(uint32_t*)(tile + (((j0 + half) >> 3) * 16 + tok) * 8 + (j0 & 7)) = hi;
    } else {
      uint16_t* tile = v_plane + ((size_t)blk * n_kv_heads + (head - n_q_heads - n_kv_heads)) * 16 * head_dim;
      tile[v_tile_off(j0, tok)] = (uint16_t)lo;
      tile[v_tile_off(j0 + 1, tok)] = (uint16_t)(lo >> 16);
      tile[v_tile_off(j0 + half, tok)] = (uint16_t)hi;
      tile[v_tile_off(j0 + half + 1, tok)] = (uint16_t)(hi >> 16);
    }
  }
};

struct ResidualEpi {
  float* resid;   // fp32 residual stream [m_pad][n], updated in place (one lane owns each element)
  int n;
  struct Row {};
  struct Pre {
    f32x4 old;
  };
  __device__ Row row_info(int) const { return Row{}; }
  __device__ Pre pre(int nb, int lane, int row, const Row&) const {
    return Pre{*(const f32x4*)(resid + resid_off(row, nb * 16 + (lane >> 4) * 4, n))};
  }
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc, const Pre& p) const {
    *(f32x4*)(resid + resid_off(row, nb * 16 + (lane >> 4) * 4, n)) = p.old + acc;
  }
};

__device__ inline float silu_f32(float z) { return z / (1.0f + __expf(-z)); }

struct SwigluEpi {
  uint16_t* hidden;  // tile layout [m_pad][ffn_k]
  int ffn_k;
  struct Row {};
  struct Pre {};
  __device__ Row row_info(int) const { return Row{}; }
  __device__ Pre pre(int, int, int, const Row&) const { return Pre{}; }
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc, const Pre&) const {
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
  // seeded sampling: 1 / temperature (0: greedy), seed, the caller's request ids (or null)
  float inv_temp;
  uint64_t seed;
  const int64_t* request_ids;
  struct Row {
    int pos, s, slot;
    uint64_t key;      // hash of (seed, request, position): the row's noise stream
  };
  typedef Row Pre;
  // output function of the splitmix64 generator
  static __device__ inline uint64_t mix(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  __device__ Row row_info(int row) const {
    Row p;
    p.pos = row_pos[row];
    p.s = row_seq[row];
    p.slot = out_logits ? dump_slot[p.s] : -1;
    p.key = 0;
    if (inv_temp != 0.f) {
      const uint64_t rid = request_ids ? (uint64_t)request_ids[p.s] : (uint64_t)p.s;
      p.key = mix(mix(seed ^ mix(rid)) ^ (uint64_t)(uint32_t)max(p.pos, 0));
    }
    return p;
  }
  __device__ Pre pre(int, int, int, const Row& r) const { return r; }
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc, const Pre& p) const {
    const int n0 = nb * 16 + (lane >> 4) * 4;
    if (out_logits && p.pos >= 0) {
      const int s = p.s, slot = p.slot;
      if (slot >= 0)
        *(f32x4*)(out_logits + ((size_t)slot * window + (row - s * window)) * vocab + n0) = acc;
    }
    // what the sampler ranks: the logits, or (temperature > 0) logit / temperature + Gumbel noise
    f32x4 val = acc;
    if (inv_temp != 0.f) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint64_t h = mix(p.key ^ (uint64_t)(n0 + e));
        const float u = (float)(2u * (uint32_t)(h >> 41) + 1u) * 0x1p-24f;   // exact: 24 significant bits, in (0, 1)
        val[e] = acc[e] * inv_temp - logf(-logf(u));
      }
    }
    // best of this lane's 4 features (ascending index, strict '>' keeps the lowest on ties) ...
    float bv = val[0];
    int bi = n0;
#pragma unroll
    for (int e = 1; e < 4; ++e)
      if (val[e] > bv) { bv = val[e]; bi = n0 + e; }
    // ... then of the 4 lanes that hold the token's other features of this block (lanes l ^ 16, l ^ 32).
    // A lane swap leaves a lane's own pair and its partner's in the two results; the rule below is
    // symmetric in the two, so every lane ends up with the same winner as with a shuffle.
    auto better_of = [](u32x2 v, u32x2 i, float& ov, int& oi) {
      const float v0 = __uint_as_float(v.x), v1 = __uint_as_float(v.y);
      const int i0 = (int)i.x, i1 = (int)i.y;
      const bool second = v1 > v0 || (v1 == v0 && i1 < i0);
      ov = second ? v1 : v0;
      oi = second ? i1 : i0;
    };
    better_of(__builtin_amdgcn_permlane16_swap(__float_as_uint(bv), __float_as_uint(bv), false, false),
              __builtin_amdgcn_permlane16_swap((uint32_t)bi, (uint32_t)bi, false, false), bv, bi);
    better_of(__builtin_amdgcn_permlane32_swap(__float_as_uint(bv), __float_as_uint(bv), false, false),
              __builtin_amdgcn_permlane32_swap((uint32_t)bi, (uint32_t)bi, false, false), bv, bi);
    if (lane < 16) amax[(size_t)row * n_blocks + nb] = make_float2(bv, __int_as_float(bi));
  }
};

// ---------------------------------------------------------------------------------------------
// Split of the reduction dimension.  A GEMM with SPLIT == 2 has TWO accumulators per output
// element: p0 over k-tiles [0, h) and p1 over k-tiles [h, k_tiles), h = (k_tiles + 1) / 2, each
// started at zero and advanced in ascending k; the result is p0 + p1 (one fp32 add).  Which GEMMs
// are split is fixed per layer type below and never depends on the number of rows.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline int split_point(int k_tiles) { return (k_tiles + 1) / 2; }

// fp32 partial of one k-half of a split GEMM (large-batch path: the halves are two launches, or the
// two y-planes of one launch, each with a buffer of its own).
struct StorePartialEpi {
  float* partial;   // [m_pad][n] in the residual-stream layout
  int n;
  size_t plane;     // distance (floats) from the first half's buffer to the second's
  struct Row {};
  struct Pre {};
  __device__ Row row_info(int) const { return Row{}; }
  __device__ Pre pre(int, int, int, const Row&) const { return Pre{}; }
  __device__ void operator()(int nb, int lane, int row, const f32x4 acc, const Pre&) const {
    *(f32x4*)(partial + resid_off(row, nb * 16 + (lane >> 4) * 4, n)) = acc;
  }
};

// Small-batch kernel for narrow outputs (at most 64 tokens): HBM-bound weight streaming with one
// workgroup per block of 16 features, so that every CU streams.  SPLIT groups of 4 waves each own
// one half of the k range.  Inside a group all 4 waves fetch the block's weight tiles, CH k-tiles
// per round (each wave every 4th tile), and park them in LDS; waves 0 .. MB-1 of the group then
// each advance one 16-token block's accumulator through the round's tiles in ascending k, with
// their own activation tiles prefetched in registers.  The next round's weight loads are issued
// before the current round is consumed.  Only the fetch is spread over the waves; the accumulation
// order per output element is the one stated above.
template <int MB, int SPLIT, class Epi>
__global__ __launch_bounds__(256 * SPLIT) void gemm_coop_kernel(const bf16x8* __restrict__ w,
                                                                const bf16x8* __restrict__ x, int k_tiles, Epi epi) {
  constexpr int CH = 32;
  __shared__ bf16x8 wlds[SPLIT][CH * 64];
  __shared__ f32x4 merge[MB][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = wave >> 2, gw = wave & 3;
  const int nb = blockIdx.x;
  const int h = SPLIT == 2 ? split_point(k_tiles) : k_tiles;
  const int k_begin = grp == 0 ? 0 : h;
  const int k_count = grp == 0 ? h : k_tiles - h;
  const int my_rounds = k_count / CH;                // full rounds of this group; the rest is the tail
  const int rounds = h / CH;                         // group 0 never has fewer than group 1
  const bf16x8* wp = w + ((size_t)nb * k_tiles + k_begin) * 64 + lane;
  const bf16x8* xp = x + ((size_t)gw * k_tiles + k_begin) * 64 + lane;   // consumer gw owns token block gw
  const bool consumer = gw < MB;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  bf16x8 wa[CH / 4], wb[CH / 4], xr[CH];
  // Weight tiles are requested two rounds ahead (register sets wa / wb alternate), activation tiles
  // one round ahead.  No load sits behind a per-load condition: the compiler would serialise them.
  auto load_w = [&](bf16x8(&dst)[CH / 4], int r) {
    const bf16x8* p = wp + (size_t)r * CH * 64;
#pragma unroll
    for (int i = 0; i < CH / 4; ++i) dst[i] = __builtin_nontemporal_load(p + (size_t)(i * 4 + gw) * 64);
  };
  auto load_x = [&](int r) {
    const bf16x8* p = xp + (size_t)r * CH * 64;
#pragma unroll
    for (int j = 0; j < CH; ++j) xr[j] = p[(size_t)j * 64];
  };
  auto round = [&](bf16x8(&cur)[CH / 4], int r) {   // consume round r (held in cur), refill cur with round r + 2
    const bool live = r < my_rounds;
    if (live) {
#pragma unroll
      for (int i = 0; i < CH / 4; ++i) wlds[grp][(i * 4 + gw) * 64 + lane] = cur[i];
    }
    __syncthreads();
    if (r + 2 < my_rounds) load_w(cur, r + 2);
    if (consumer && live) {
#pragma unroll
      for (int j = 0; j < CH; ++j) acc = mfma16(wlds[grp][j * 64 + lane], xr[j], acc);
      if (r + 1 < my_rounds) load_x(r + 1);
    }
    __syncthreads();
  };
  if (my_rounds > 0) {
    load_w(wa, 0);
    if (consumer) load_x(0);
  }
  if (my_rounds > 1) load_w(wb, 1);
  typename Epi::Pre pre{};
  if (consumer && grp == 0) pre = epi.pre(nb, lane, gw * 16 + (lane & 15), epi.row_info(gw * 16 + (lane & 15)));
  for (int r = 0; r < rounds; r += 2) {
    round(wa, r);
    if (r + 1 < rounds) round(wb, r + 1);
  }
  if (consumer) {   // tail of fewer than CH tiles (model dimensions that are no multiple of 1024): tile by tile
    for (int kt = my_rounds * CH; kt < k_count; ++kt) acc = mfma16(wp[(size_t)kt * 64], xp[(size_t)kt * 64], acc);
  }
  if (SPLIT == 2) {
    if (consumer && grp == 1) merge[gw][lane] = acc;
    __syncthreads();
    if (consumer && grp == 0) acc = acc + merge[gw][lane];
  }
  if (consumer && grp == 0) epi(nb, lane, gw * 16 + (lane & 15), acc, pre);
}

// Small-batch kernel for wide outputs (at most 64 tokens): 8 waves per workgroup, every wave owns
// its own block of 16 features and streams that block's weight tiles from HBM into registers, 16
// k-tiles ahead of their use.  The activation tiles, which all 8 waves need, are fetched
// once per workgroup and shared through LDS (double buffered), which cuts the L2 traffic for
// activations by 8.  Accumulation order per output element: as stated above.  A round is 16 k-tiles
// for one or two token blocks and 8 for four (three register sets of weights then), so that the
// registers hold the accumulators, the weights in flight and a few prefetched activation operands.
// (The same kernel with 8 and 16 token blocks only ties the tiled kernel at 128 and 256 rows: a round's
// arithmetic then outlasts neither the weight stream nor the latency of its own activation fetch.)
// NBW (7 or 8) of the 8 waves own a feature block; with NBW = 7 the eighth wave only helps fetching
// activations (this makes the grid of the 8B gate/up GEMM exactly one workgroup per CU).
template <int MB, int NBW, class Epi>
__global__ __launch_bounds__(512) void gemm_xshare_kernel(const bf16x8* __restrict__ w, const bf16x8* __restrict__ x,
                                                          int n_blocks, int k_tiles, Epi epi) {
  // A round is CH k-tiles; NSET register sets of weights: one in use, NSET - 1 in flight (16 KiB per
  // wave whatever the round length).  The round's activation tiles go through LDS, double buffered.
  constexpr int CH = MB <= 2 ? 16 : MB <= 8 ? 8 : 4, NSET = 16 / CH + 1, NW = 8;
  constexpr int XT = MB * CH / NW;                   // activation tiles each wave fetches per round
  static_assert(MB * CH % NW == 0, "a round's activation tiles are dealt evenly to the waves");
  __shared__ bf16x8 xlds[2][MB * CH * 64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const bool owner = wave < NBW && blockIdx.x * NBW + wave < n_blocks;   // other waves only fetch activations
  const int nb = owner ? blockIdx.x * NBW + wave : 0;
  const bf16x8* wp = w + (size_t)nb * k_tiles * 64 + lane;
  const bf16x8* xp = x + lane;
  f32x4 acc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b) acc[b] = (f32x4){0.f, 0.f, 0.f, 0.f};
  bf16x8 wr[NSET][CH], xg[XT];
  const int rounds = k_tiles / CH;                   // full rounds; the rest is the tail

  // none of these loads sits behind a per-load condition (the compiler would serialise them)
  // (a round past the last one re-reads the last round's first tile CH times: loads that keep the
  // loop free of branches but fetch next to nothing from HBM)
  auto load_w = [&](bf16x8(&dst)[CH], int r) {
    const int real = r < rounds ? 1 : 0, base = min(r, rounds - 1) * CH;
#pragma unroll
    for (int j = 0; j < CH; ++j) dst[j] = __builtin_nontemporal_load(wp + (size_t)(base + j * real) * 64);
  };
  auto load_x = [&](int r) {   // tile q of the round: token block q / CH, k-tile r * CH + q % CH
#pragma unroll
    for (int i = 0; i < XT; ++i) {
      const int q = i * NW + wave;
      xg[i] = xp[((size_t)(q / CH) * k_tiles + r * CH + q % CH) * 64];
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XT; ++i) xlds[buf][(i * NW + wave) * 64 + lane] = xg[i];
  };
  auto compute = [&](const bf16x8(&cur)[CH], int buf) __attribute__((always_inline)) {
    if constexpr (MB <= 2) {
#pragma unroll
      for (int j = 0; j < CH; ++j)
#pragma unroll
        for (int b = 0; b < MB; ++b) acc[b] = mfma16(cur[j], xlds[buf][(b * CH + j) * 64 + lane], acc[b]);
    } else {
      // many token blocks: the activation operands are requested from LDS PD MFMAs ahead, by hand
      // (with the registers this full, the compiler reads each operand right before its MFMA)
      constexpr int PD = 6, N = CH * MB;
      bf16x8 xq[PD + 1];
      auto operand = [&](int idx) { return xlds[buf][((idx % MB) * CH + idx / MB) * 64 + lane]; };
#pragma unroll
      for (int t = 0; t < PD; ++t) xq[t] = operand(t);
#pragma unroll
      for (int idx = 0; idx < N; ++idx) {
        if (idx + PD < N) xq[(idx + PD) % (PD + 1)] = operand(idx + PD);
        __builtin_amdgcn_sched_barrier(0);
        acc[idx % MB] = mfma16(cur[idx / MB], xq[idx % (PD + 1)], acc[idx % MB]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // what the epilogue needs from memory: requested now (hidden behind the weight stream) while the
  // registers allow it, at the end with 4 token blocks and more
  constexpr bool kEarlyPre = MB < 4;
  typename Epi::Pre pre[kEarlyPre ? MB : 1];
  if (kEarlyPre && owner) {
#pragma unroll
    for (int b = 0; b < MB; ++b) pre[b] = epi.pre(nb, lane, b * 16 + (lane & 15), epi.row_info(b * 16 + (lane & 15)));
  }
  // A round's body is free of branches: past the last round the loads re-read the last round (into
  // registers and a buffer that nothing uses any more).  The activation loads of a round are issued
  // BEFORE its weight loads: loads return in order, so the wait for the activations (they go to LDS
  // within the round) then leaves the weight loads, which are needed NSET - 1 rounds later, in flight.
  // Rounds come in groups of NSET without an exit in between (with one, the compiler moves a round's
  // weight loads down to the round that uses them, which serialises fetch and arithmetic); the last
  // rounds % NSET rounds follow as straight code.
  auto run = [&](auto own) __attribute__((always_inline)) {
    constexpr bool OWN = decltype(own)::value;
    const int last = rounds - 1;
    load_x(0);
    if (OWN) {
#pragma unroll
      for (int u = 0; u < NSET - 1; ++u) load_w(wr[u], u);
    }
    store_x(0);
    __syncthreads();
    int flip = 0;                                    // activation buffer of the current round (NSET odd)
    auto body = [&](auto uc, int rr) __attribute__((always_inline)) {
      constexpr int u = decltype(uc)::value;
      const int buf = NSET % 2 == 0 ? (u & 1) : flip;
      load_x(min(rr + 1, last));
      // the set that the previous round used up takes the round NSET - 1 ahead
      if (OWN) load_w(wr[(u + NSET - 1) % NSET], rr + NSET - 1);
      __builtin_amdgcn_sched_barrier(0);             // (left alone the compiler sinks the loads behind the round's MFMAs)
      if (OWN) compute(wr[u], buf);
      store_x(buf ^ 1);
      __syncthreads();
      flip ^= 1;
    };
    int r = 0;
    for (; r + NSET <= rounds; r += NSET) {
      body(std::integral_constant<int, 0>{}, r);
      body(std::integral_constant<int, 1>{}, r + 1);
      if constexpr (NSET > 2) body(std::integral_constant<int, 2>{}, r + 2);
      if constexpr (NSET > 3) body(std::integral_constant<int, 3>{}, r + 3);
      if constexpr (NSET > 4) body(std::integral_constant<int, 4>{}, r + 4);
    }
    if (r < rounds) body(std::integral_constant<int, 0>{}, r);
    if (r + 1 < rounds) body(std::integral_constant<int, 1>{}, r + 1);
    if constexpr (NSET > 3) {
      if (r + 2 < rounds) body(std::integral_constant<int, 2>{}, r + 2);
    }
    if constexpr (NSET > 4) {
      if (r + 3 < rounds) body(std::integral_constant<int, 3>{}, r + 3);
    }
  };
  static_assert(NSET >= 2 && NSET <= 5, "the groups of rounds are written out for 2 .. 5 register sets");
  if (rounds > 0) {
    if (owner) run(std::true_type{});
    else run(std::false_type{});
  }
  for (int kt = rounds * CH; owner && kt < k_tiles; ++kt) {   // tail of fewer than CH tiles: tile by tile
    const bf16x8 a = wp[(size_t)kt * 64];
#pragma unroll
    for (int b = 0; b < MB; ++b) acc[b] = mfma16(a, xp[((size_t)b * k_tiles + kt) * 64], acc[b]);
  }
  if (owner) {
#pragma unroll
    for (int b = 0; b < MB; ++b) {
      const int row = b * 16 + (lane & 15);
      if constexpr (kEarlyPre) epi(nb, lane, row, acc[b], pre[b]);
      else epi(nb, lane, row, acc[b], epi.pre(nb, lane, row, epi.row_info(row)));
    }
  }
}

// Large-batch kernel (more than 64 tokens): MFMA-bound, LDS-tiled.  A workgroup of 2*WN waves (WN along
// the features x 2 along the tokens; WN = 2 unless stated) owns a tile of 16*WN*WBN features x 32*WBM
// tokens; each wave owns WBN x WBM MFMA blocks (WBN*WBM*4
// accumulator registers).  Per stage of one k-tile the waves move the tile's WN*WBN + 2*WBM operand
// tiles (1 KiB each, already in MFMA operand order) from global memory straight into a ring of NST
// stages in LDS; every wave reads its WBN weight operands and WBM activation operands per k-tile
// with conflict-free 16-byte LDS reads.  WGS workgroups share a CU: one wave per SIMD cannot keep
// the MFMA pipe busy by itself (an MFMA loop on registers alone reaches 58 % of peak with one wave
// per SIMD and 89 % with two), so the shipped shape is 128 x 256 with two workgroups per CU.
// Workgroups are numbered so that the workgroups that land on one XCD (id mod 8) form super-tiles
// of up to 32 neighbouring tiles (shape and size chosen per launch, see launch_tiled): weight and
// activation tiles are then fetched from HBM once per XCD and served from that XCD's L2 to the rest
// of the super-tile.
// Accumulation order per output element: k ascending inside [k_begin, k_begin + k_count), exactly
// as in the small-batch kernels; with ADD_PARTIAL the other half's fp32 partial is added at the end.
// 1 KiB from global memory (wave-uniform `base` + per-lane byte offset `voff`) straight into LDS at
// byte address `dst` + 16 * lane (M0 holds the wave-uniform destination).  Written as assembly on
// purpose: with the compiler's own form of this load every later LDS read waits for all earlier
// ones, which un-pipelines the operand reads.  The compiler therefore does not count these loads;
// lds_fetch_wait() is the only wait that covers them.  Nothing else in these kernels uses M0.
__device__ __forceinline__ void lds_fetch_1k(const void* base, uint32_t voff, uint32_t dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(dst) : "memory", "m0");
}
// acc += a * b with the accumulator pinned to the same four accumulation registers before and after.
// (Left to the compiler, some instantiations of the tiled kernel compute into a temporary and copy
// it back - four moves behind every MFMA of the main loop.)  The compiler does not know that this is
// an MFMA: the kernel leaves idle cycles between its last MFMA and the first read of an accumulator
// (mfma_drain), and never issues two of these on the same accumulator back to back.
__device__ __forceinline__ void mfma16_inplace(const bf16x8 a, const bf16x8 b, f32x4& acc) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

// At most N of the fetches this wave has issued are still on their way (they complete in order).
template <int N>
__device__ __forceinline__ void lds_fetch_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

template <int WBN, int WBM, int NST, int WGS, bool ADD_PARTIAL, class Epi, int WN = 2>
__global__ __launch_bounds__(128 * WN, WGS) void gemm_tiled_kernel(const bf16x8* __restrict__ w, const bf16x8* __restrict__ x,
                                                         int n_blocks, int k_tiles, int k_begin, int k_count,
                                                         const float* __restrict__ partial, int n, int tiles_n,
                                                         int tiles_m, int sm_tiles, int group_tiles, int planes, Epi epi) {
  constexpr int TBN = WN * WBN, TBM = 2 * WBM;  // 16-row blocks per tile side (features, tokens)
  constexpr int ST = TBN + TBM;                 // operand tiles per stage of one k-tile (weights then activations)
  constexpr int NWV = 2 * WN;                   // waves per workgroup: WN along the features x 2 along the tokens
  constexpr int PW = (ST + NWV - 1) / NWV;      // operand tiles each wave fetches per stage (where ST is no multiple of
                                                // the wave count the last waves fetch the stage's last tile again: the same
                                                // bytes to the same place, which keeps every wave's fetch count the same)
  // NST = ring of stages in LDS
  __shared__ bf16x8 lds[NST][ST * 64];
  // wave index as a scalar, so that everything derived from it (operand addresses) stays in SGPRs
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wn = wave >> 1, wm = wave & 1;
  // XCD-aware numbering.  Workgroup ids are dealt round-robin to the 8 XCDs; G consecutive ids of one
  // XCD form a super-tile of SN feature tiles x SM token tiles (SN * SM = G), so that per k-step the
  // XCD's L2 fetches SN weight tiles + SM activation tiles for G workgroups.  Super-tiles are dealt
  // to the XCDs round-robin; the two k-halves of a side-by-side split are numbered one after the other.
  // G is 32 when that still gives every XCD a super-tile, less for small launches; SM follows the
  // number of token tiles.  (A workgroup without a tile still has to wait for a CU with free LDS
  // before it can leave, so holes in the numbering are expensive.)
  const int G = group_tiles, SM = sm_tiles, SN = G / SM;
  const int sup_n = (tiles_n + SN - 1) / SN, sup_m = (tiles_m + SM - 1) / SM;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int sup_all = (local / G) * 8 + xcd, in_sup = local % G;
  const int plane = sup_all / (sup_n * sup_m), sup = sup_all % (sup_n * sup_m);
  if (plane >= planes) return;
  const int tn = (sup / sup_m) * SN + in_sup / SM, tm = (sup % sup_m) * SM + in_sup % SM;
  if (tn >= tiles_n || tm >= tiles_m) return;
  const int n0 = tn * TBN, m0 = tm * TBM;      // first feature / token block of the tile
  if constexpr (std::is_same<Epi, StorePartialEpi>::value) {
    // both halves of a split GEMM in one launch: plane 1 takes the k-tiles after the first k_count
    if (plane) {
      k_begin = k_count;
      k_count = k_tiles - k_count;
      epi.partial += epi.plane;
    }
  }

  // Operand tiles go from global memory straight into LDS (no staging registers, no LDS stores):
  // per stage this wave moves PW tiles of 1 KiB, lane i's 16 bytes landing at tile base + 16 i.
  // src[i] is the wave-uniform start of the i-th tile's row block (k-tile k_begin).
  const bf16x8* src[PW];
#pragma unroll
  for (int i = 0; i < PW; ++i) {
    const int q = min(wave * PW + i, ST - 1);          // 0 .. ST-1
    const bool is_w = q < TBN;
    const int blk = is_w ? q : q - TBN;
    const int gb = is_w ? min(n0 + blk, n_blocks - 1) : m0 + blk;   // feature blocks past the matrix re-read the last one
    src[i] = (is_w ? w : x) + ((size_t)gb * k_tiles + k_begin) * 64;
  }
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&lds[0][0];
  auto fetch = [&](int s) {      // k-tiles past the range re-read the last one
    const uint32_t voff = (uint32_t)min(s, k_count - 1) * 1024u + (uint32_t)lane * 16u;
#pragma unroll
    for (int i = 0; i < PW; ++i)
      lds_fetch_1k(src[i], voff, lds_addr + (uint32_t)(((s % NST) * ST + min(wave * PW + i, ST - 1)) * 1024));
  };
  f32x4 acc[WBN][WBM];
#pragma unroll
  for (int i = 0; i < WBN; ++i)
#pragma unroll
    for (int j = 0; j < WBM; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // One stage = one k-tile = WBM groups of WBN MFMAs (group j: token block j against the wave's WBN
  // feature blocks).  Software pipelined by hand across stages, so that the MFMA pipe never waits for
  // LDS or for the barrier: the activation operand of a group is requested from LDS PD groups ahead,
  // and after group JB - when every read of this stage has been issued - the wave waits for the next
  // stage's tiles, meets the others, refills the ring slot this stage occupied and requests the next
  // stage's weight operands, all while the remaining groups of this stage still run.  (The scheduling
  // barriers keep the compiler from sinking the reads next to their uses.)
  constexpr int PD = 3, JB = WBM - PD;
  static_assert(WBM % (PD + 1) == 0 && JB >= 0, "operand ring must line up across stages");
  bf16x8 bq[PD + 1];
  auto w_operands = [&](bf16x8(&dst)[WBN], int s) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < WBN; ++i) dst[i] = lds[s % NST][(wn * WBN + i) * 64 + lane];
  };
  auto x_operand = [&](int s, int j) { return lds[s % NST][(TBN + wm * WBM + j) * 64 + lane]; };
  // The loop body is kept free of branches (the register allocation of 256 accumulators does not
  // survive control flow inside it): every stage issues a fetch and waits with the same count.  Past
  // the end of the k range the fetches re-read the last k-tile into ring slots that nothing reads.
#pragma unroll
  for (int s = 0; s < NST; ++s) fetch(s);
  lds_fetch_wait<(NST - 1) * PW>();                    // stage 0 has landed
  __syncthreads();
#pragma unroll
  for (int t = 0; t < PD; ++t) bq[t] = x_operand(0, t);
  bf16x8 a[2][WBN];
  w_operands(a[0], 0);
  auto stage = [&](int s, const bf16x8(&cur)[WBN], bf16x8(&next)[WBN]) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < WBM; ++j) {
      if (j == JB) {
        lds_fetch_wait<(NST - 2) * PW>();              // stage s + 1 has landed: only the two after it may be outstanding
        __syncthreads();                               // also: every wave has read all it needs of stage s
        fetch(s + NST);                                // into the slot of stage s
        w_operands(next, s + 1);                       // weight operands of the next stage, while this one finishes
      }
      // (in the last stage the operands requested for a following stage are stale tiles that nothing consumes)
      bq[(j + PD) % (PD + 1)] = j + PD < WBM ? x_operand(s, j + PD) : x_operand(s + 1, j + PD - WBM);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < WBN; ++i) mfma16_inplace(cur[i], bq[j % (PD + 1)], acc[i][j]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  {
    int s = 0;
    for (; s + 1 < k_count; s += 2) {
      stage(s, a[0], a[1]);
      stage(s + 1, a[1], a[0]);
    }
    if (s < k_count) stage(s, a[0], a[1]);
  }
  lds_fetch_wait<0>();
  mfma_drain();
  // epilogue, token block by token block: what depends on the token row only is fetched once per row
#pragma unroll
  for (int j = 0; j < WBM; ++j) {
    const int row = (m0 + wm * WBM + j) * 16 + (lane & 15);
    const typename Epi::Row ri = epi.row_info(row);
#pragma unroll
    for (int i = 0; i < WBN; ++i) {
      const int nb = n0 + wn * WBN + i;
      if (nb < n_blocks) {
        f32x4 v = acc[i][j];
        if (ADD_PARTIAL) v = v + *(const f32x4*)(partial + resid_off(row, nb * 16 + (lane >> 4) * 4, n));
        epi(nb, lane, row, v, epi.pre(nb, lane, row, ri));
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // one token block at a time: hoisting the next blocks' loads up here costs spills
  }
}

// p0 + p1 of a split GEMM whose halves ran side by side, handed to the GEMM's epilogue with the
// same (feature block, lane, row) ownership as in the GEMM kernels: one wave per 16 x 16 block.
template <class Epi>
__global__ __launch_bounds__(256) void split_combine_kernel(const float* __restrict__ p0, const float* __restrict__ p1,
                                                            int n_blocks, int n, Epi epi) {
  const int lane = threadIdx.x & 63;
  const int nb = blockIdx.x * 4 + (threadIdx.x >> 6), row = blockIdx.y * 16 + (lane & 15);
  if (nb >= n_blocks) return;
  const size_t off = resid_off(row, nb * 16 + (lane >> 4) * 4, n);
  const typename Epi::Pre pre = epi.pre(nb, lane, row, epi.row_info(row));
  const f32x4 v = *(const f32x4*)(p0 + off) + *(const f32x4*)(p1 + off);
  epi(nb, lane, row, v, pre);
}

// side_by_side (split GEMMs only): both k-halves in one launch of twice the workgroups plus a small
// combining pass, instead of two launches one after the other - for launches that do not fill the
// device by themselves.  The arithmetic per output element is the same either way.
template <int WBN, int WBM, int NST, int WGS, int SPLIT, class Epi, int WN = 2>
void launch_tiled(const bf16x8* wp, const bf16x8* xp, int n_blocks, int k_tiles, int n, const Workspace& ws,
                  const Epi& epi, hipStream_t st, bool side_by_side = false) {
  const int tiles_n = (n_blocks + WN * WBN - 1) / (WN * WBN), tiles_m = ws.m_pad / (32 * WBM);
  constexpr unsigned threads = 128 * WN;
  const int planes = SPLIT == 2 && side_by_side ? 2 : 1;
  // Super-tiles of g = sn x sm tiles (see the kernel), dealt round-robin to the 8 XCDs.  sm: as square as the tiles
  // allow (a 128 x 256 tile counts double on the token side), but the widest that leaves at most 15 % of the token
  // columns empty - a ragged last column of super-tiles is workgroups without a tile, and those still queue for a CU
  // with free LDS before they can leave (1280 rows took as long as 2048 that way; a column of width 1 on the other
  // hand makes every XCD fetch 32 weight tiles per k-step, which cost 4 % at 1792 rows).  g: the largest of 32, 16, 8, 4 that leaves
  // the busiest XCD within 3 % of the least workgroup slots any of them gives it (few super-tiles deal out unevenly).
  const int sm_max = 2 * WBM > WN * WBN ? 4 : 8;
  int g = 4, sm = 1, sn = 4, supers = 0;
  long long least = -1;
  for (int pass = 0; pass < 2; ++pass)
    for (int cand = 32; cand >= 4; cand /= 2) {
      int csm = 1;
      for (int w = 2; w <= sm_max && w <= cand; w *= 2) {
        const int padded = (tiles_m + w - 1) / w * w;
        if ((padded - tiles_m) * 100 <= padded * 15) csm = w;
      }
      const int csn = cand / csm;
      const int csupers = ((tiles_n + csn - 1) / csn) * ((tiles_m + csm - 1) / csm) * planes;
      const long long per_xcd = (long long)((csupers + 7) / 8) * cand;
      if (pass == 0) {
        if (least < 0 || per_xcd < least) least = per_xcd;
      } else if (per_xcd * 100 <= least * 103) {
        g = cand, sm = csm, sn = csn, supers = csupers;
        pass = 2;   // (the largest that qualifies: leave both loops)
        break;
      }
    }
  const unsigned grid = 8u * (unsigned)g * (unsigned)((supers + 7) / 8);
  if (SPLIT == 1) {
    gemm_tiled_kernel<WBN, WBM, NST, WGS, false, Epi, WN><<<grid, threads, 0, st>>>(wp, xp, n_blocks, k_tiles, 0, k_tiles,
                                                                                    nullptr, n, tiles_n, tiles_m, sm, g, 1, epi);
    return;
  }
  const int h = split_point(k_tiles);
  const size_t plane = (size_t)ws.m_pad * n;
  StorePartialEpi pe{ws.split_part, n, plane};
  if (side_by_side) {
    gemm_tiled_kernel<WBN, WBM, NST, WGS, false, StorePartialEpi, WN><<<grid, threads, 0, st>>>(
        wp, xp, n_blocks, k_tiles, 0, h, nullptr, n, tiles_n, tiles_m, sm, g, 2, pe);
    split_combine_kernel<Epi><<<dim3((n_blocks + 3) / 4, ws.m_pad / 16), 256, 0, st>>>(ws.split_part, ws.split_part + plane,
                                                                                      n_blocks, n, epi);
  } else {
    gemm_tiled_kernel<WBN, WBM, NST, WGS, false, StorePartialEpi, WN><<<grid, threads, 0, st>>>(
        wp, xp, n_blocks, k_tiles, h, k_tiles - h, nullptr, n, tiles_n, tiles_m, sm, g, 1, pe);
    gemm_tiled_kernel<WBN, WBM, NST, WGS, true, Epi, WN><<<grid, threads, 0, st>>>(wp, xp, n_blocks, k_tiles, 0, h, ws.split_part,
                                                                                   n, tiles_n, tiles_m, sm, g, 1, epi);
  }
}

#ifndef LLM42_TILE_BIG
#define LLM42_TILE_BIG 4, 8, 3, 2
#endif
enum GemmKind { GEMM_QKV = 0, GEMM_RESIDUAL = 1, GEMM_GATE_UP = 2, GEMM_LOGITS = 3 };
// The split of each GEMM type (part of the reduction schedule, see above).
constexpr int kSplit[4] = {1, 2, 1, 1};

template <int SPLIT, class Epi>
void launch_gemm(const uint16_t* w, const uint16_t* x, int n_blocks, int k_padded, int n, const Workspace& ws,
                 bool wide, const Epi& epi, hipStream_t st) {
  const int k_tiles = k_padded / 32, m_pad = ws.m_pad;
  const bf16x8* wp = (const bf16x8*)w;
  const bf16x8* xp = (const bf16x8*)x;
  if (m_pad <= 64) {
    if (wide && SPLIT == 1) {
      // 7 or 8 feature blocks per workgroup: whichever needs less (rounds of 256 workgroups) x (blocks each)
      const int g8 = (n_blocks + 7) / 8, g7 = (n_blocks + 6) / 7;
      const bool seven = ((g7 + 255) / 256) * 7 < ((g8 + 255) / 256) * 8;
      const unsigned gx = (unsigned)(seven ? g7 : g8);
      if (seven) {
        if (m_pad == 16) gemm_xshare_kernel<1, 7, Epi><<<gx, 512, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
        else if (m_pad == 32) gemm_xshare_kernel<2, 7, Epi><<<gx, 512, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
        else gemm_xshare_kernel<4, 7, Epi><<<gx, 512, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
      } else {
        if (m_pad == 16) gemm_xshare_kernel<1, 8, Epi><<<gx, 512, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
        else if (m_pad == 32) gemm_xshare_kernel<2, 8, Epi><<<gx, 512, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
        else gemm_xshare_kernel<4, 8, Epi><<<gx, 512, 0, st>>>(wp, xp, n_blocks, k_tiles, epi);
      }
    } else {
      if (m_pad == 16) gemm_coop_kernel<1, SPLIT, Epi><<<n_blocks, 256 * SPLIT, 0, st>>>(wp, xp, k_tiles, epi);
      else if (m_pad == 32) gemm_coop_kernel<2, SPLIT, Epi><<<n_blocks, 256 * SPLIT, 0, st>>>(wp, xp, k_tiles, epi);
      else gemm_coop_kernel<4, SPLIT, Epi><<<n_blocks, 256 * SPLIT, 0, st>>>(wp, xp, k_tiles, epi);
    }
    return;
  }
  // More than 64 tokens: m_pad is 128, 256 or 512, or a multiple of 256 beyond that.  Larger tiles
  // move fewer operand bytes per flop, smaller ones give more workgroups; measured over 128 .. 4096 rows
  // of the 8B shapes, the best choice is the largest tile that still yields about as many workgroups as
  // the device has CUs.  Where the epilogue is heavy (rotary embedding and cache writes) the 128 x 256
  // tile waits until it fills the device, since its epilogues overlap less with other workgroups' main
  // loops; the LM head never takes it.  A split GEMM runs its halves side by side unless each half
  // fills the device by itself.
  const long long cus = ws.num_cus;
  const long long t256 = m_pad % 256 == 0 ? (long long)((n_blocks + 7) / 8) * (m_pad / 256) : 0;
  const long long t128 = (long long)((n_blocks + 7) / 8) * (m_pad / 128);
  const bool side_by_side = SPLIT == 2 && t256 < 2 * cus;
  const int p = side_by_side ? 2 : 1;
  constexpr bool kLogits = std::is_same<Epi, LogitsEpi>::value, kQkv = std::is_same<Epi, QkvEpi>::value;
  const bool big = !kLogits && (kQkv ? t256 >= 2 * cus : t256 * p * 5 >= 4 * cus);
  if constexpr (!std::is_same<Epi, SwigluEpi>::value) {
    // 768 and 1024 rows (and 1280 of the QKV projection): too few 128 x 256 tiles for two workgroups per CU, and one
    // workgroup of four waves per CU keeps neither the MFMA pipe nor the fetch path busy.  The same tile with EIGHT
    // waves (32 x 128 per wave, one workgroup per CU, six stages in flight) measured 3 - 13 % faster on these
    // launches (not on gate/up, whose 128 x 128 tiles already fill the device twice over).
    if (m_pad == 768 || m_pad == 1024 || (kQkv && m_pad == 1280)) {
      launch_tiled<2, 8, 6, 1, SPLIT, Epi, 4>(wp, xp, n_blocks, k_tiles, n, ws, epi, st, side_by_side);
      return;
    }
  }
  if constexpr (kQkv) {
    // A 192 x 128 tile where it puts the whole QKV projection into one round of workgroups (two per CU) and the
    // 128 x 128 tile would need a second one: 2048 rows of the 8B shape are 512 such tiles (3.67 -> 3.24 ms per pass).
    const long long t192 = (long long)((n_blocks + 11) / 12) * (m_pad / 128);
    // ... and where 192 x 128 tiles make whole rounds and 128 x 256 tiles do not (4096 rows: 1024 against 768 tiles,
    // 6.20 -> 6.10 ms per pass; 6144 rows: 9.54 -> 8.85).
    const bool whole_rounds = n_blocks % 12 == 0 && t192 % (2 * cus) == 0 && t256 % (2 * cus) != 0;
    if (whole_rounds || (!big && n_blocks % 12 == 0 && t192 <= 2 * cus && t128 > 2 * cus)) {
      launch_tiled<6, 4, 4, 2, SPLIT, Epi>(wp, xp, n_blocks, k_tiles, n, ws, epi, st, false);
      return;
    }
  }
  if (big)
    launch_tiled<LLM42_TILE_BIG, SPLIT, Epi>(wp, xp, n_blocks, k_tiles, n, ws, epi, st, side_by_side);
  else if (t128 * p * 4 >= 3 * cus)
    launch_tiled<4, 4, 4, 2, SPLIT, Epi>(wp, xp, n_blocks, k_tiles, n, ws, epi, st, side_by_side);
  else
    launch_tiled<2, 4, 12, 1, SPLIT, Epi>(wp, xp, n_blocks, k_tiles, n, ws, epi, st, side_by_side);
}

}  // namespace

void launch_gemm_qkv(const llm42_model* m, int layer, const llm42_kv_cache* kv, int window, const Workspace& ws,
                     hipStream_t st) {
  const llm42_config& c = m->cfg;
  const size_t plane = (size_t)kv->num_blocks * c.n_kv_heads * 16 * c.head_dim;
  QkvEpi e;
  e.row_rope = (const float4*)ws.row_rope;
  e.row_pos = ws.row_pos;
  e.row_seq = ws.row_seq;
  e.row_blk = ws.row_blk;
  e.q = ws.q;
  e.k_plane = (uint16_t*)kv->kv_base + ((size_t)layer * 2 + 0) * plane;
  e.v_plane = (uint16_t*)kv->kv_base + ((size_t)layer * 2 + 1) * plane;
  e.n_q_heads = c.n_q_heads;
  e.n_kv_heads = c.n_kv_heads;
  e.head_dim = c.head_dim;
  e.group = m->group;
  e.window = window;
  e.r_pad = ws.r_pad;
  launch_gemm<kSplit[GEMM_QKV]>(m->layers[layer].wqkv, ws.normed, m->n_qkv / 16, c.d_model, m->n_qkv, ws, false, e, st);
}

void launch_gemm_residual(const uint16_t* w, const uint16_t* x, float* resid, int n, int k_padded,
                          const Workspace& ws, hipStream_t st) {
  ResidualEpi e{resid, n};
  // Off the fixed schedule (fast path, cost-of-determinism measurement) the split follows the batch,
  // as in an ordinary engine: two halves while there are few rows to spread over the device, none beyond.
  if (ws.batch_chosen && ws.m_rows > 16) launch_gemm<1>(w, x, n / 16, k_padded, n, ws, false, e, st);
  else launch_gemm<kSplit[GEMM_RESIDUAL]>(w, x, n / 16, k_padded, n, ws, false, e, st);
}

void launch_gemm_swiglu(const llm42_model* m, int layer, const Workspace& ws, hipStream_t st) {
  SwigluEpi e{ws.hidden, m->ffn_k};
  launch_gemm<kSplit[GEMM_GATE_UP]>(m->layers[layer].wgu, ws.normed, m->gu_blocks, m->cfg.d_model, m->gu_blocks * 16, ws, true, e, st);
}

void launch_gemm_logits(const llm42_model* m, int window, float* out_logits, const llm42_sampling* sampling,
                        const Workspace& ws, hipStream_t st) {
  LogitsEpi e;
  e.row_pos = ws.row_pos;
  e.row_seq = ws.row_seq;
  e.dump_slot = ws.dump_slot;
  e.out_logits = out_logits;
  e.amax = ws.amax;
  e.window = window;
  e.vocab = m->cfg.vocab;
  e.n_blocks = m->cfg.vocab / 16;
  const bool sampled = sampling && sampling->temperature > 0.f;
  e.inv_temp = sampled ? 1.0f / sampling->temperature : 0.f;
  e.seed = sampled ? sampling->seed : 0;
  e.request_ids = sampled ? sampling->request_ids : nullptr;
  launch_gemm<kSplit[GEMM_LOGITS]>(m->lm_head, ws.normed, m->cfg.vocab / 16, m->cfg.d_model, m->cfg.vocab, ws, true, e, st);
}
