// C ABI of the verifier library (declared in include/llm42.h): host-side
// validation, model construction, workspace carving and the kernel sequence of
// one verifier pass.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "llm42_dev.h"

// Scratch area of llm42_verify_window_static: one copy per GPU that loads the library, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; the device address it yields (one per
// device) is what kernels, copies and fills are given.
static __device__ __align__(256) unsigned char scratch[LLM42_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, set by llm42_model_create
std::mutex g_scratch_mutex;

thread_local char g_err[512] = "";

llm42_status fail(llm42_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail(LLM42_EHIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

// ---- optional per-launch timing (a measurement aid, off by default) -------------------------
struct Profiler {
  int kind = -2;                       // -2 off, -1 every kernel class, >= 0 one class
  std::vector<hipEvent_t> ev;          // pairs (start, stop)
  std::vector<int32_t> kinds;
  size_t used = 0;                     // events recorded so far
} g_prof;

struct ScopedEvent {
  hipStream_t st;
  bool on;
  ScopedEvent(int kind, hipStream_t s) : st(s), on(false) {
    if (g_prof.kind == -2 || (g_prof.kind >= 0 && g_prof.kind != kind) || g_prof.used + 2 > g_prof.ev.size()) return;
    on = true;
    g_prof.kinds[g_prof.used / 2] = kind;
    (void)hipEventRecord(g_prof.ev[g_prof.used], st);
  }
  ~ScopedEvent() {
    if (!on) return;
    (void)hipEventRecord(g_prof.ev[g_prof.used + 1], st);
    g_prof.used += 2;
  }
};
#define TIMED(kind, call)        \
  do {                           \
    ScopedEvent se_(kind, st);   \
    call;                        \
  } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int pad_to(int x, int a) { return (x + a - 1) / a * a; }

llm42_status check_config(const llm42_config& c) {
  if (c.n_layers < 1 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.d_ffn < 1 || c.vocab < 1 ||
      c.max_position < 1)
    return fail(LLM42_EINVAL, "config: non-positive dimension");
  if (!(c.rope_theta > 0.f) || !(c.rms_eps >= 0.f)) return fail(LLM42_EINVAL, "config: bad rope_theta / rms_eps");
  if (c.kv_block_size != LLM42_KV_BLOCK) return fail(LLM42_ESHAPE, "config: kv_block_size must be 16");
  if (c.head_dim != 64 && c.head_dim != 128) return fail(LLM42_ESHAPE, "config: head_dim must be 64 or 128");
  if (c.d_model % 128) return fail(LLM42_ESHAPE, "config: d_model must be a multiple of 128");
  if (c.d_ffn % 16 || c.vocab % 16) return fail(LLM42_ESHAPE, "config: d_ffn and vocab must be multiples of 16");
  if (c.d_ffn < 64) return fail(LLM42_ESHAPE, "config: d_ffn must be at least 64 (each half of the split down-projection needs a k-tile)");
  if (c.n_q_heads % c.n_kv_heads || c.n_q_heads / c.n_kv_heads > 8)
    return fail(LLM42_ESHAPE, "config: n_q_heads must be 1..8 times n_kv_heads");
  return LLM42_OK;
}

// How the attention work of a call is split (work distribution only; the bits do not depend on it).
void attention_mode(const llm42_model* m, int num_seqs, int max_context, Workspace& ws) {
  const llm42_config& c = m->cfg;
  // attention work split: per chunk while the grid would otherwise be small, per super beyond that
  const int col_blocks = ws.r_pad / 16, cb_groups = (col_blocks + (col_blocks >= 8 ? 8 : 4) - 1) / (col_blocks >= 8 ? 8 : 4);
  // One workgroup per 2048-key super (chunks folded in registers) once that gives enough workgroups - measured at
  // 8 .. 32 sequences and contexts 512 .. 6000: from about 192 (pairs x supers) on it beats one workgroup per chunk
  // plus the merge of 8 x as many partials.  Contexts that all fit one super need no merge pass at all (the
  // attention kernel normalises and writes the output itself), which pays from 128 workgroups on.
  // With two or more such workgroups per CU and contexts beyond one super the call may instead take whole sequences
  // as items: one workgroup walks all supers of a (sequence, kv head), folds them in registers in the merge pass's
  // order and writes the output (the store instructions that end a work item interrupt the workgroup's fetch stream,
  // and a super's fp32 partial takes nine per wave where a whole sequence's bf16 rows take four).  Whether the
  // sequences of the call deal out evenly enough for that is decided on the device, by the plan kernel.
  const long long pairs = (long long)num_seqs * c.n_kv_heads * cb_groups;
  const int supers = attention_units(true, max_context);
  ws.attn_seq = col_blocks >= 8 && supers > 1 && pairs >= 2LL * ws.num_cus;
  ws.attn_direct = supers == 1 && pairs >= 128;
  ws.attn_super = ws.attn_direct || pairs * supers >= 192;
  ws.attn_units = attention_units(ws.attn_super, max_context);
}

// Carve the workspace.  Called with base == nullptr to size it.
Workspace carve(const llm42_model* m, int num_seqs, int window, int max_context, char* base, bool batch_chosen = false,
                size_t min_part_rows = 0) {
  const llm42_config& c = m->cfg;
  Workspace ws;
  memset(&ws, 0, sizeof ws);
  ws.num_cus = m->num_cus;
  ws.batch_chosen = batch_chosen;
  ws.m_rows = num_seqs * window;
  // (384 padded rows would be three token tiles of 128: too few for the 128 x 128 tile to fill the device, and the
  // 64 x 128 tile then needs a second round of workgroups - 512 padded rows run faster than 384)
  ws.m_pad = ws.m_rows <= 16 ? 16 : ws.m_rows <= 32 ? 32 : ws.m_rows <= 64 ? 64
             : ws.m_rows <= 256 ? pad_to(ws.m_rows, 128) : ws.m_rows <= 512 ? 512 : pad_to(ws.m_rows, 256);
  ws.r_pad = pad_to(m->group * window, 16);
  attention_mode(m, num_seqs, max_context, ws);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off = align_up(off + bytes, 256);
    return p;
  };
  ws.row_pos = (int32_t*)take(sizeof(int32_t) * ws.m_pad);
  ws.row_seq = (int32_t*)take(sizeof(int32_t) * ws.m_pad);
  ws.seq_len = (int32_t*)take(sizeof(int32_t) * num_seqs);
  ws.seq_n = (int32_t*)take(sizeof(int32_t) * num_seqs);
  ws.dump_slot = (int32_t*)take(sizeof(int32_t) * num_seqs);
  ws.row_blk = (int32_t*)take(sizeof(int32_t) * ws.m_pad);
  ws.row_rope = (float2*)take(sizeof(float2) * (size_t)ws.m_pad * (c.head_dim / 2));
  ws.resid = (float*)take(4ull * ws.m_pad * c.d_model);
  ws.normed = (uint16_t*)take(2ull * ws.m_pad * c.d_model);
  ws.q = (uint16_t*)take(2ull * num_seqs * c.n_kv_heads * ws.r_pad * c.head_dim);
  ws.attn = (uint16_t*)take(2ull * ws.m_pad * m->d_attn);
  ws.hidden = (uint16_t*)take(2ull * ws.m_pad * m->ffn_k);
  // (min_part_rows: llm42_workspace_bytes sizes the partials for every call of up to max_seqs sequences - a call of
  // fewer sequences may run per chunk where the largest runs per super, with 8 x the slots per sequence)
  const size_t part_rows = std::max((size_t)num_seqs * c.n_kv_heads * ws.attn_units * ws.r_pad, min_part_rows);
  ws.part_acc = (float*)take(4ull * part_rows * c.head_dim);
  ws.part_ml = (float*)take(8ull * part_rows);
  ws.attn_items = (int4*)take(sizeof(int4) * std::max((size_t)num_seqs * ws.attn_units, min_part_rows / ((size_t)c.n_kv_heads * ws.r_pad)));
  ws.attn_ctrl_offset = off;
  ws.attn_ctrl = (int32_t*)take(sizeof(int32_t) * (2 + c.n_layers));
  ws.amax = (float2*)take(8ull * ws.m_pad * (c.vocab / 16));
  ws.split_part = (float*)take(ws.m_pad > 64 ? 2 * 4ull * ws.m_pad * c.d_model : 0);
  ws.bytes = off;
  return ws;
}

// Bytes that serve every call of 1 .. max_seqs sequences: everything but the attention partials grows with the
// number of sequences; the partials depend on the work split as well (a few sequences run per 256-key chunk where many
// run per 2048-key super), so their slots are counted for every n.
size_t sized_for_up_to(const llm42_model* m, int max_seqs, int window, int max_context) {
  Workspace w;
  memset(&w, 0, sizeof w);
  w.num_cus = m->num_cus;
  w.r_pad = pad_to(m->group * window, 16);
  size_t part_rows = 0;
  for (int n = 1; n <= max_seqs; ++n) {
    attention_mode(m, n, max_context, w);
    part_rows = std::max(part_rows, (size_t)n * m->cfg.n_kv_heads * w.attn_units * w.r_pad);
  }
  return carve(m, max_seqs, window, max_context, nullptr, false, part_rows).bytes;
}

// One pass of the verifier over num_seqs x window rows; arguments already checked.
llm42_status run_pass(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens, const int32_t* candidates,
                      int window, const int32_t* n_valid, int num_seqs, int max_context, int32_t* out_tokens,
                      int32_t* seq_status, float* out_logits, const int32_t* dump_seq_ids, int n_dump,
                      const Workspace& ws, hipStream_t st, const llm42_sampling* sampling, bool prefill_pass) {
  const llm42_config& c = m->cfg;
  TIMED(LLM42_K_PREPARE, launch_prepare(m, kv, seq_lens, candidates, n_valid, num_seqs, window, max_context,
                                        dump_seq_ids, n_dump, out_tokens, seq_status, ws, st, prefill_pass));
  TIMED(LLM42_K_PREPARE, launch_attention_plan(m, num_seqs, max_context, ws, st));
  TIMED(LLM42_K_EMBED, launch_embed(m, candidates, ws, st));
  for (int l = 0; l < c.n_layers; ++l) {
    const llm42_model::Layer& ly = m->layers[l];
    TIMED(LLM42_K_RMSNORM, launch_rmsnorm(ws.resid, ly.attn_norm, ws.normed, ws.m_pad, c.d_model, c.rms_eps, st));
    TIMED(LLM42_K_QKV, launch_gemm_qkv(m, l, kv, window, ws, st));
    TIMED(LLM42_K_ATTENTION, launch_attention(m, l, kv, num_seqs, window, max_context, ws, st));
    TIMED(LLM42_K_O_PROJ, launch_gemm_residual(ly.wo, ws.attn, ws.resid, c.d_model, m->d_attn, ws, st));
    TIMED(LLM42_K_RMSNORM, launch_rmsnorm(ws.resid, ly.ffn_norm, ws.normed, ws.m_pad, c.d_model, c.rms_eps, st));
    TIMED(LLM42_K_GATE_UP, launch_gemm_swiglu(m, l, ws, st));
    TIMED(LLM42_K_DOWN, launch_gemm_residual(ly.wdown, ws.hidden, ws.resid, c.d_model, m->ffn_k, ws, st));
  }
  TIMED(LLM42_K_RMSNORM, launch_rmsnorm(ws.resid, m->final_norm, ws.normed, ws.m_pad, c.d_model, c.rms_eps, st));
  TIMED(LLM42_K_LM_HEAD, launch_gemm_logits(m, window, out_logits, sampling, ws, st));
  TIMED(LLM42_K_ARGMAX, launch_argmax_merge(m, num_seqs, window, out_tokens, ws, st));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LLM42_EHIP, "verifier pass: launch failed: %s", hipGetErrorString(e));
  return LLM42_OK;
}

// Buffers of llm42_prefill behind the verifier's own workspace: the candidate rows of the current
// pass, their count and the cached length per sequence, the pass's tokens, a status word per sequence.
struct PrefillExtra {
  int32_t *cand, *n_valid, *lens_now, *pass_tokens, *status;
  size_t bytes;   // workspace size including these
};
PrefillExtra carve_prefill(size_t verifier_bytes, int num_seqs, int window, char* base) {
  PrefillExtra x;
  size_t off = align_up(verifier_bytes, 256);
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off = align_up(off + bytes, 256);
    return (int32_t*)p;
  };
  x.cand = take(sizeof(int32_t) * (size_t)num_seqs * window);
  x.n_valid = take(sizeof(int32_t) * num_seqs);
  x.lens_now = take(sizeof(int32_t) * num_seqs);
  x.pass_tokens = take(sizeof(int32_t) * (size_t)num_seqs * window);
  x.status = take(sizeof(int32_t) * num_seqs);
  x.bytes = off;
  return x;
}

// llm42_verify_window_sampled and llm42_decode_step_sampled behind their argument names; batch_chosen: see Workspace.
llm42_status verify_impl(const char* who, const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                         const int32_t* candidates, int32_t window, const int32_t* n_valid, int32_t num_seqs,
                         int32_t max_context, int32_t* out_tokens, int32_t* seq_status, float* out_logits,
                         const int32_t* dump_seq_ids, int32_t n_dump, void* workspace, size_t workspace_bytes,
                         void* hip_stream, const llm42_sampling* sampling, bool batch_chosen) {
  if (sampling && !(sampling->temperature >= 0.f)) return fail(LLM42_EINVAL, "%s: negative temperature", who);
  if (!m || !kv || !seq_lens || !candidates || !out_tokens || !workspace)
    return fail(LLM42_EINVAL, "%s: null argument", who);
  if (!kv->kv_base || !kv->block_table || kv->num_blocks < 1 || kv->max_blocks_per_seq < 1)
    return fail(LLM42_EINVAL, "%s: bad kv_cache view", who);
  if (window < 1 || window > LLM42_MAX_WINDOW) return fail(LLM42_EINVAL, "%s: window must be 1..%d", who, LLM42_MAX_WINDOW);
  if (num_seqs < 1 || (int64_t)num_seqs * window > LLM42_MAX_ROWS)
    return fail(LLM42_EINVAL, "%s: num_seqs * window must be 1..%d", who, LLM42_MAX_ROWS);
  if (n_dump < 0 || (n_dump > 0 && (!out_logits || !dump_seq_ids)))
    return fail(LLM42_EINVAL, "%s: n_dump needs out_logits and dump_seq_ids", who);
  if (max_context < 1) return fail(LLM42_EINVAL, "%s: max_context < 1", who);
  if (max_context > m->cfg.max_position)
    return fail(LLM42_ECAPACITY, "%s: max_context %d exceeds max_position %d", who, max_context, m->cfg.max_position);
  if ((int64_t)max_context > (int64_t)kv->max_blocks_per_seq * LLM42_KV_BLOCK)
    return fail(LLM42_ECAPACITY, "%s: max_context %d exceeds block-table capacity %lld", who, max_context,
                (long long)kv->max_blocks_per_seq * LLM42_KV_BLOCK);
  if ((uintptr_t)workspace % 256) return fail(LLM42_EWORKSPACE, "%s: workspace not 256-byte aligned", who);
  const Workspace ws = carve(m, num_seqs, window, max_context, (char*)workspace, batch_chosen);
  if (ws.bytes > workspace_bytes)
    return fail(LLM42_EWORKSPACE, "%s: workspace %zu < %zu bytes", who, workspace_bytes, ws.bytes);
  return run_pass(m, kv, seq_lens, candidates, window, n_valid, num_seqs, max_context, out_tokens, seq_status,
                  n_dump > 0 ? out_logits : nullptr, dump_seq_ids, n_dump, ws, (hipStream_t)hip_stream, sampling, false);
}

}  // namespace

extern "C" {

const char* llm42_last_error(void) { return g_err; }

const char* llm42_schedule_info(void) {
  return "llm42-gfx950 0.2; gemm: v_mfma_f32_16x16x32_bf16, k ascending, split_k=2 (halves, p0+p1) for the two residual projections, 1 elsewhere; "
         "attention: step=64 keys, chunk=256, super=2048, left folds, a partial's reference exponent moves when a step's maximum exceeds it by more than 8 (log2); "
         "rmsnorm: 16x4 partial sums per row";
}

llm42_status llm42_model_create(const llm42_config* cfg, const llm42_weights* w, llm42_model** out) {
  if (!cfg || !w || !out) return fail(LLM42_EINVAL, "model_create: null argument");
  *out = nullptr;
  if (llm42_status st = check_config(*cfg)) return st;
  if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
      !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
    return fail(LLM42_EINVAL, "model_create: null weight pointer");
  const llm42_config& c = *cfg;
  for (int l = 0; l < c.n_layers; ++l)
    if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate[l] ||
        !w->w_up[l] || !w->w_down[l])
      return fail(LLM42_EINVAL, "model_create: null weight pointer in layer %d", l);

  llm42_model* m = new llm42_model();
  m->cfg = c;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
      delete m;
      return fail(LLM42_EHIP, "model_create: cannot query the device");
    }
    m->num_cus = cus;
    m->device = dev;
    // the address of this device's copy of the built-in scratch area (looked up once per device, here, with the
    // device current; llm42_verify_window_static only reads the table)
    if (dev < kMaxDevices) {
      std::lock_guard<std::mutex> lock(g_scratch_mutex);
      if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t se = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (se != hipSuccess || !ptr) {
          delete m;
          return fail(LLM42_EHIP, "model_create: hipGetSymbolAddress(scratch): %s", hipGetErrorString(se));
        }
        g_scratch_ptr[dev] = ptr;
      }
    }
  }
  m->group = c.n_q_heads / c.n_kv_heads;
  m->n_qkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  m->d_attn = c.n_q_heads * c.head_dim;
  m->ffn_k = pad_to(c.d_ffn, 32);
  m->gu_blocks = m->ffn_k / 8;
  m->layers = new llm42_model::Layer[c.n_layers];

  // one arena: sizes in bf16 elements, every piece 256-byte aligned
  const size_t d = c.d_model;
  const size_t sz_embed = (size_t)c.vocab * d, sz_norm = align_up(d, 128), sz_lm = (size_t)c.vocab * d;
  const size_t sz_qkv = (size_t)m->n_qkv * d, sz_o = d * m->d_attn, sz_gu = (size_t)m->gu_blocks * 16 * d,
               sz_down = d * m->ffn_k;
  const size_t per_layer = 2 * sz_norm + sz_qkv + sz_o + sz_gu + sz_down;
  const size_t rope_bytes = (size_t)c.max_position * (c.head_dim / 2) * 2 * sizeof(float);
  const size_t elems = sz_embed + sz_norm + sz_lm + per_layer * c.n_layers;
  m->arena_bytes = align_up(elems * 2, 256) + rope_bytes;
  hipError_t e = hipMalloc((void**)&m->arena, m->arena_bytes);
  if (e != hipSuccess) {
    const size_t wanted = m->arena_bytes;
    delete[] m->layers;
    delete m;
    return fail(LLM42_EHIP, "model_create: hipMalloc(%zu): %s", wanted, hipGetErrorString(e));
  }
  uint16_t* p = m->arena;
  auto take = [&](size_t n) {
    uint16_t* r = p;
    p += n;
    return r;
  };
  m->embed = take(sz_embed);
  m->final_norm = take(sz_norm);
  m->lm_head = take(sz_lm);
  hipStream_t st = nullptr;
  auto copy = [&](uint16_t* dst, const void* src, size_t n) {
    return hipMemcpyAsync(dst, src, n * 2, hipMemcpyDeviceToDevice, st);
  };
  hipError_t ce = copy(m->embed, w->embed, sz_embed);
  if (ce == hipSuccess) ce = copy(m->final_norm, w->final_norm, d);
  launch_pack_plain((const uint16_t*)w->lm_head, m->lm_head, c.vocab, c.d_model, c.d_model, st);
  for (int l = 0; l < c.n_layers && ce == hipSuccess; ++l) {
    llm42_model::Layer& ly = m->layers[l];
    ly.attn_norm = take(sz_norm);
    ly.ffn_norm = take(sz_norm);
    ly.wqkv = take(sz_qkv);
    ly.wo = take(sz_o);
    ly.wgu = take(sz_gu);
    ly.wdown = take(sz_down);
    ce = copy(ly.attn_norm, w->attn_norm[l], d);
    if (ce == hipSuccess) ce = copy(ly.ffn_norm, w->ffn_norm[l], d);
    launch_pack_qkv((const uint16_t*)w->wq[l], (const uint16_t*)w->wk[l], (const uint16_t*)w->wv[l], ly.wqkv, c, st);
    launch_pack_plain((const uint16_t*)w->wo[l], ly.wo, c.d_model, m->d_attn, m->d_attn, st);
    launch_pack_gate_up((const uint16_t*)w->w_gate[l], (const uint16_t*)w->w_up[l], ly.wgu, c.d_ffn, m->gu_blocks,
                        c.d_model, st);
    launch_pack_plain((const uint16_t*)w->w_down[l], ly.wdown, c.d_model, c.d_ffn, m->ffn_k, st);
  }
  // rotary table: angle = pos * theta^(-2j/head_dim), evaluated in double, stored as fp32 (cos, sin)
  m->rope = (float*)((char*)m->arena + align_up(elems * 2, 256));
  if (ce == hipSuccess) {
    const int half = c.head_dim / 2;
    std::vector<float> tab((size_t)c.max_position * half * 2);
    std::vector<double> inv_freq(half);
    for (int j = 0; j < half; ++j) inv_freq[j] = std::pow((double)c.rope_theta, -2.0 * j / c.head_dim);
    for (int pos = 0; pos < c.max_position; ++pos)
      for (int j = 0; j < half; ++j) {
        const double a = pos * inv_freq[j];
        tab[((size_t)pos * half + j) * 2 + 0] = (float)std::cos(a);
        tab[((size_t)pos * half + j) * 2 + 1] = (float)std::sin(a);
      }
    ce = hipMemcpy(m->rope, tab.data(), rope_bytes, hipMemcpyHostToDevice);
  }
  if (ce == hipSuccess) ce = hipGetLastError();
  if (ce == hipSuccess) ce = hipStreamSynchronize(st);
  if (ce != hipSuccess) {
    llm42_model_destroy(m);
    return fail(LLM42_EHIP, "model_create: %s", hipGetErrorString(ce));
  }
  *out = m;
  return LLM42_OK;
}

void llm42_model_destroy(llm42_model* m) {
  if (!m) return;
  if (m->arena) (void)hipFree(m->arena);
  delete[] m->layers;
  delete m;
}

llm42_status llm42_kv_bytes(const llm42_model* m, int64_t num_blocks, size_t* out_bytes) {
  if (!m || !out_bytes || num_blocks < 0) return fail(LLM42_EINVAL, "kv_bytes: bad argument");
  *out_bytes = (size_t)m->cfg.n_layers * 2 * (size_t)num_blocks * m->cfg.n_kv_heads * 16 * m->cfg.head_dim * 2;
  return LLM42_OK;
}

llm42_status llm42_workspace_bytes(const llm42_model* m, int32_t max_seqs, int32_t window, int32_t max_context,
                                   size_t* out_bytes) {
  if (!m || !out_bytes) return fail(LLM42_EINVAL, "workspace_bytes: null argument");
  if (max_seqs < 1 || window < 1 || window > LLM42_MAX_WINDOW || max_context < 1)
    return fail(LLM42_EINVAL, "workspace_bytes: max_seqs/window/max_context out of range");
  if ((int64_t)max_seqs * window > LLM42_MAX_ROWS)
    return fail(LLM42_EINVAL, "workspace_bytes: more than %d rows", LLM42_MAX_ROWS);
  *out_bytes = sized_for_up_to(m, max_seqs, window, max_context);
  return LLM42_OK;
}

llm42_status llm42_verify_window(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                                 const int32_t* candidates, int32_t window, const int32_t* n_valid, int32_t num_seqs,
                                 int32_t max_context, int32_t* out_tokens, int32_t* seq_status, float* out_logits,
                                 const int32_t* dump_seq_ids, int32_t n_dump, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  return llm42_verify_window_sampled(m, kv, seq_lens, candidates, window, n_valid, num_seqs, max_context, out_tokens,
                                     seq_status, out_logits, dump_seq_ids, n_dump, workspace, workspace_bytes,
                                     hip_stream, nullptr);
}

llm42_status llm42_verify_window_sampled(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                                         const int32_t* candidates, int32_t window, const int32_t* n_valid,
                                         int32_t num_seqs, int32_t max_context, int32_t* out_tokens,
                                         int32_t* seq_status, float* out_logits, const int32_t* dump_seq_ids,
                                         int32_t n_dump, void* workspace, size_t workspace_bytes, void* hip_stream,
                                         const llm42_sampling* sampling) {
  return verify_impl("verify_window", m, kv, seq_lens, candidates, window, n_valid, num_seqs, max_context, out_tokens,
                     seq_status, out_logits, dump_seq_ids, n_dump, workspace, workspace_bytes, hip_stream, sampling,
                     false);
}

llm42_status llm42_measure_verify_window_batch_chosen(const llm42_model* m, const llm42_kv_cache* kv,
                                                      const int32_t* seq_lens, const int32_t* candidates,
                                                      int32_t window, const int32_t* n_valid, int32_t num_seqs,
                                                      int32_t max_context, int32_t* out_tokens, int32_t* seq_status,
                                                      float* out_logits, const int32_t* dump_seq_ids, int32_t n_dump,
                                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  return verify_impl("measure_verify_window_batch_chosen", m, kv, seq_lens, candidates, window, n_valid, num_seqs,
                     max_context, out_tokens, seq_status, out_logits, dump_seq_ids, n_dump, workspace, workspace_bytes,
                     hip_stream, nullptr, true);
}

llm42_status llm42_measure_attention_plan(const llm42_model* m, int32_t num_seqs, int32_t window, int32_t max_context,
                                          int64_t* out) {
  if (!m || !out) return fail(LLM42_EINVAL, "measure_attention_plan: null argument");
  if (num_seqs < 1 || window < 1 || window > LLM42_MAX_WINDOW || max_context < 1 ||
      (int64_t)num_seqs * window > LLM42_MAX_ROWS)
    return fail(LLM42_EINVAL, "measure_attention_plan: num_seqs/window/max_context out of range");
  const Workspace ws = carve(m, num_seqs, window, max_context, nullptr);
  out[0] = ws.attn_super ? 2048 : 256;
  out[1] = ws.attn_direct ? 1 : 0;
  out[2] = ws.attn_seq ? 1 : 0;
  out[3] = (int64_t)(ws.attn_ctrl_offset + sizeof(int32_t) * (1 + m->cfg.n_layers));
  out[4] = ws.r_pad / 16 >= 8 ? 1 : 0;
  return LLM42_OK;
}

llm42_status llm42_verify_window_static(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                                        const int32_t* candidates, int32_t window, const int32_t* n_valid,
                                        int32_t num_seqs, int32_t max_context, int32_t* out_tokens,
                                        int32_t* seq_status, float* out_logits, const int32_t* dump_seq_ids,
                                        int32_t n_dump, void* hip_stream) {
  if (!m) return fail(LLM42_EINVAL, "verify_window_static: null argument");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != m->device)
    return fail(LLM42_EINVAL, "verify_window_static: the model lives on device %d, current device is %d", m->device, dev);
  void* ptr = dev >= 0 && dev < kMaxDevices ? g_scratch_ptr[dev] : nullptr;
  if (!ptr) return fail(LLM42_EHIP, "verify_window_static: no scratch address for device %d", dev);
  if (window >= 1 && window <= LLM42_MAX_WINDOW && num_seqs >= 1 && (int64_t)num_seqs * window <= LLM42_MAX_ROWS &&
      max_context >= 1) {
    const size_t need = carve(m, num_seqs, window, max_context, nullptr).bytes;
    if (need > LLM42_STATIC_SCRATCH_BYTES)
      return fail(LLM42_EWORKSPACE, "verify_window_static: this call needs %zu bytes of scratch, the built-in area holds %zu",
                  need, (size_t)LLM42_STATIC_SCRATCH_BYTES);
  }
  return verify_impl("verify_window_static", m, kv, seq_lens, candidates, window, n_valid, num_seqs, max_context,
                     out_tokens, seq_status, out_logits, dump_seq_ids, n_dump, ptr, LLM42_STATIC_SCRATCH_BYTES, hip_stream,
                     nullptr, false);
}

llm42_status llm42_decode_step(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                               const int32_t* tokens, int32_t num_seqs, int32_t max_context, int32_t* out_tokens,
                               int32_t* seq_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return llm42_decode_step_sampled(m, kv, seq_lens, tokens, num_seqs, max_context, out_tokens, seq_status, workspace,
                                   workspace_bytes, hip_stream, nullptr);
}

llm42_status llm42_decode_step_sampled(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                                       const int32_t* tokens, int32_t num_seqs, int32_t max_context,
                                       int32_t* out_tokens, int32_t* seq_status, void* workspace,
                                       size_t workspace_bytes, void* hip_stream, const llm42_sampling* sampling) {
  return verify_impl("decode_step", m, kv, seq_lens, tokens, 1, nullptr, num_seqs, max_context, out_tokens, seq_status,
                     nullptr, nullptr, 0, workspace, workspace_bytes, hip_stream, sampling, true);
}

llm42_status llm42_prefill_workspace_bytes(const llm42_model* m, int32_t max_seqs, int32_t chunk, int32_t max_context,
                                           size_t* out_bytes) {
  size_t v = 0;
  if (!out_bytes) return fail(LLM42_EINVAL, "prefill_workspace_bytes: null argument");
  if (llm42_status st = llm42_workspace_bytes(m, max_seqs, chunk, max_context, &v)) return st;
  *out_bytes = carve_prefill(v, max_seqs, chunk, nullptr).bytes;
  return LLM42_OK;
}

llm42_status llm42_prefill(const llm42_model* m, const llm42_kv_cache* kv, const int32_t* seq_lens,
                           const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t num_seqs,
                           int32_t max_prompt_len, int32_t chunk, int32_t max_context, int32_t* out_next_tokens,
                           int32_t* seq_status, void* workspace, size_t workspace_bytes, void* hip_stream,
                           const llm42_sampling* sampling) {
  if (sampling && !(sampling->temperature >= 0.f)) return fail(LLM42_EINVAL, "prefill: negative temperature");
  if (!m || !kv || !seq_lens || !prompt_tokens || !prompt_offsets || !out_next_tokens || !workspace)
    return fail(LLM42_EINVAL, "prefill: null argument");
  if (!kv->kv_base || !kv->block_table || kv->num_blocks < 1 || kv->max_blocks_per_seq < 1)
    return fail(LLM42_EINVAL, "prefill: bad kv_cache view");
  if (chunk < 1 || chunk > LLM42_MAX_WINDOW) return fail(LLM42_EINVAL, "prefill: chunk must be 1..%d", LLM42_MAX_WINDOW);
  if (num_seqs < 1 || (int64_t)num_seqs * chunk > LLM42_MAX_ROWS)
    return fail(LLM42_EINVAL, "prefill: num_seqs * chunk must be 1..%d", LLM42_MAX_ROWS);
  if (max_prompt_len < 0 || max_context < 1) return fail(LLM42_EINVAL, "prefill: bad max_prompt_len / max_context");
  if (max_context > m->cfg.max_position)
    return fail(LLM42_ECAPACITY, "prefill: max_context %d exceeds max_position %d", max_context, m->cfg.max_position);
  if ((int64_t)max_context > (int64_t)kv->max_blocks_per_seq * LLM42_KV_BLOCK)
    return fail(LLM42_ECAPACITY, "prefill: max_context %d exceeds block-table capacity %lld", max_context,
                (long long)kv->max_blocks_per_seq * LLM42_KV_BLOCK);
  if ((uintptr_t)workspace % 256) return fail(LLM42_EWORKSPACE, "prefill: workspace not 256-byte aligned");
  const Workspace ws = carve(m, num_seqs, chunk, max_context, (char*)workspace);
  const PrefillExtra x = carve_prefill(ws.bytes, num_seqs, chunk, (char*)workspace);
  if (x.bytes > workspace_bytes) return fail(LLM42_EWORKSPACE, "prefill: workspace %zu < %zu bytes", workspace_bytes, x.bytes);
  hipStream_t st = (hipStream_t)hip_stream;
  int32_t* status = seq_status ? seq_status : x.status;
  const int passes = max_prompt_len == 0 ? 1 : (max_prompt_len + chunk - 1) / chunk;   // one pass at least: it sets the outputs
  for (int p = 0; p < passes; ++p) {
    launch_prefill_window(prompt_tokens, prompt_offsets, seq_lens, num_seqs, chunk, p, max_prompt_len, x.cand, x.n_valid,
                          x.lens_now, status, out_next_tokens, st);
    if (max_prompt_len == 0) break;
    if (llm42_status rc = run_pass(m, kv, x.lens_now, x.cand, chunk, x.n_valid, num_seqs, max_context, x.pass_tokens, status,
                                   nullptr, nullptr, 0, ws, st, sampling, true))
      return rc;
    launch_prefill_pick(prompt_offsets, num_seqs, chunk, p, x.pass_tokens, status, out_next_tokens, st);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LLM42_EHIP, "prefill: launch failed: %s", hipGetErrorString(e));
  return LLM42_OK;
}

llm42_status llm42_commit_rollback(const int32_t* candidates, const int32_t* out_tokens, const int32_t* n_valid,
                                   int32_t num_seqs, int32_t window, int32_t* seq_lens, int32_t* committed_counts,
                                   int32_t* committed_tokens, int32_t* rolled_back_counts, void* hip_stream) {
  if (!candidates || !out_tokens || !seq_lens || !committed_counts || !committed_tokens)
    return fail(LLM42_EINVAL, "commit_rollback: null argument");
  if (num_seqs < 1 || window < 1 || window > LLM42_MAX_WINDOW)
    return fail(LLM42_EINVAL, "commit_rollback: num_seqs/window out of range");
  hipStream_t st = (hipStream_t)hip_stream;
  TIMED(LLM42_K_COMMIT, launch_commit(candidates, out_tokens, n_valid, num_seqs, window, seq_lens, committed_counts,
                                      committed_tokens, rolled_back_counts, st));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LLM42_EHIP, "commit_rollback: launch failed: %s", hipGetErrorString(e));
  return LLM42_OK;
}

llm42_status llm42_profile_enable(int32_t kind, int32_t max_launches) {
  if (kind < -1 || kind >= LLM42_K_COUNT || max_launches < 1 || max_launches > (1 << 20))
    return fail(LLM42_EINVAL, "profile_enable: bad kind or max_launches");
  while (g_prof.ev.size() < 2 * (size_t)max_launches) {
    hipEvent_t e;
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) return fail(LLM42_EHIP, "profile_enable: hipEventCreate: %s", hipGetErrorString(err));
    g_prof.ev.push_back(e);
  }
  g_prof.kinds.assign(g_prof.ev.size() / 2, -1);
  g_prof.used = 0;
  g_prof.kind = kind;
  return LLM42_OK;
}

llm42_status llm42_profile_collect(float* ms_out, int32_t* kinds_out, int32_t capacity, int32_t* n_out) {
  if (!ms_out || !n_out || capacity < 0) return fail(LLM42_EINVAL, "profile_collect: bad argument");
  const size_t n = g_prof.used / 2;
  g_prof.kind = -2;
  *n_out = 0;
  for (size_t i = 0; i < n && (int32_t)i < capacity; ++i) {
    hipError_t err = hipEventSynchronize(g_prof.ev[2 * i + 1]);
    if (err == hipSuccess) err = hipEventElapsedTime(&ms_out[i], g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
    if (err != hipSuccess) return fail(LLM42_EHIP, "profile_collect: %s", hipGetErrorString(err));
    if (kinds_out) kinds_out[i] = g_prof.kinds[i];
    *n_out = (int32_t)i + 1;
  }
  g_prof.used = 0;
  return LLM42_OK;
}

}  // extern "C"
