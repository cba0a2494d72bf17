/* llm42.h -- C ABI of the MI355X (gfx950) verifier library for LLM-42's
 * decode-verify-rollback protocol.
 *
 * The library implements the verifier side of the protocol [paper Section 4.2]:
 *   llm42_verify_window   replays a fixed window of tokens per sequence (one
 *                         consistent token followed by candidates from the fast
 *                         path) through a decoder-only transformer in one causal
 *                         pass, overwrites the window's KV-cache entries with its
 *                         own [Section 4.2 "Making KV cache consistent"] and
 *                         returns the greedy token after every input
 *                         [Section 4.4 "Sampling": arg-max, lowest index on ties];
 *   llm42_commit_rollback applies the accept rule [Section 4.2 Case-1, Case-2]:
 *                         longest reproduced prefix of candidates plus the
 *                         verifier's own next token; KV length truncated there.
 *
 * Every floating-point reduction runs under a schedule that depends only on the
 * model's dimensions and on the token's absolute position in its own sequence,
 * never on how many sequences or rows the call holds or where a sequence sits
 * in the batch: each logit is bitwise identical for any batch size, batch
 * composition, batch slot and split of the positions into windows.  (The paper
 * obtains this from off-the-shelf kernels by fixing the input shape
 * [Section 4.1 "Leveraging O2"]; here it holds by construction, so groups of any
 * size [Section 4.3] may be verified together.)
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on the current HIP device;
 *     "host" pointers are ordinary process memory.
 *   - All matrices handed to llm42_model_create are bf16, row-major,
 *     [out_features][in_features].
 *   - Hot calls (verify_window, commit_rollback) allocate nothing, never
 *     synchronise and never read device memory on the host: they validate the
 *     host-visible arguments, enqueue kernels on `hip_stream` and return.
 *   - Return value: LLM42_OK or a negative llm42_status; llm42_last_error()
 *     returns a host string describing the last failure on the calling thread.
 */
#ifndef LLM42_H_
#define LLM42_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t llm42_status;
#define LLM42_OK           0
#define LLM42_EINVAL      -1  /* null pointer, negative size, window < 1, ...            */
#define LLM42_ESHAPE      -2  /* model dimensions the kernels do not support              */
#define LLM42_EWORKSPACE  -3  /* workspace too small or misaligned (256 B)                */
#define LLM42_ECAPACITY   -4  /* max_context exceeds block-table or position capacity     */
#define LLM42_EHIP        -5  /* a HIP call or kernel launch failed                       */

#define LLM42_KV_BLOCK 16     /* tokens per KV-cache block; the only supported value      */
#define LLM42_MAX_WINDOW 512  /* largest verification window (the window ablation of SS 5.3 spans 16 .. 512) */
#define LLM42_MAX_ROWS 65536  /* most rows (num_seqs * window) of one call; beyond it the calls return LLM42_EINVAL */

/* Per-sequence status bits written to `seq_status` by llm42_verify_window. */
#define LLM42_SEQ_OK            0
#define LLM42_SEQ_BAD_LENGTH    1  /* seq_len < 0, n_valid outside 1..window, or seq_len + n_valid > max_context */
#define LLM42_SEQ_BAD_BLOCK     2  /* a needed block-table entry is < 0 or >= num_blocks  */
#define LLM42_SEQ_BAD_TOKEN     4  /* an input token id is outside [0, vocab)             */

typedef struct llm42_model llm42_model;  /* opaque; owns repacked device weights + RoPE table */

/* Model dimensions (caller-owned POD).  Supported: head_dim in {64, 128};
 * d_model a multiple of 128; d_ffn, vocab multiples of 16;
 * n_q_heads a multiple of n_kv_heads with ratio <= 8; kv_block_size == 16. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float   rope_theta;      /* rotary base; pairing (j, j + head_dim/2), no frequency rescaling */
  float   rms_eps;
  int32_t kv_block_size;   /* LLM42_KV_BLOCK */
  int32_t max_position;    /* rotary table length: positions 0 .. max_position-1 are usable   */
} llm42_config;

/* Plain weights, all DEVICE pointers to bf16 row-major matrices.  Arrays with
 * one entry per layer are HOST arrays of device pointers.  The library copies
 * (repacks) everything during llm42_model_create; the caller may free the
 * originals afterwards. */
typedef struct {
  const void* embed;              /* [vocab][d_model]                         */
  const void* final_norm;         /* [d_model]                                */
  const void* lm_head;            /* [vocab][d_model]                         */
  const void* const* attn_norm;   /* per layer [d_model]                      */
  const void* const* wq;          /* per layer [n_q_heads*head_dim][d_model]  */
  const void* const* wk;          /* per layer [n_kv_heads*head_dim][d_model] */
  const void* const* wv;          /* per layer [n_kv_heads*head_dim][d_model] */
  const void* const* wo;          /* per layer [d_model][n_q_heads*head_dim]  */
  const void* const* ffn_norm;    /* per layer [d_model]                      */
  const void* const* w_gate;      /* per layer [d_ffn][d_model]               */
  const void* const* w_up;        /* per layer [d_ffn][d_model]               */
  const void* const* w_down;      /* per layer [d_model][d_ffn]               */
} llm42_weights;

/* Paged KV cache: a view of caller-owned device memory.
 *
 * kv_base holds n_layers * 2 * num_blocks * n_kv_heads tiles of
 * 16 * head_dim bf16 values, indexed [layer][0 = K, 1 = V][block][kv_head].
 * Inside a tile (token t = position % 16, feature f):
 *   K tile: element index ((f / 8) * 16 + t) * 8 + f % 8     (8-feature groups, token-minor)
 *   V tile: element index (((f / 16) * 4 + t / 4) * 16 + f % 16) * 4 + t % 4
 *                                         (16-feature blocks, 4-token groups, feature, token-minor)
 * Position p of sequence s lives in block block_table[s][p / 16].
 * llm42_kv_bytes() gives the size of the whole cache. */
typedef struct {
  void*          kv_base;             /* dev                                              */
  int64_t        num_blocks;          /* physical blocks per (layer, K|V) plane           */
  const int32_t* block_table;         /* dev [num_seqs][max_blocks_per_seq] physical ids  */
  int32_t        max_blocks_per_seq;
} llm42_kv_cache;

/* Build a model: validates cfg (LLM42_ESHAPE), allocates device memory for the
 * repacked weights and the rotary table, repacks on the current device, and
 * synchronises once.  The model belongs to the caller until llm42_model_destroy. */
llm42_status llm42_model_create(const llm42_config* cfg, const llm42_weights* weights, llm42_model** out);
void         llm42_model_destroy(llm42_model* model);

/* Bytes of KV cache for `num_blocks` blocks (all layers, K and V). */
llm42_status llm42_kv_bytes(const llm42_model* model, int64_t num_blocks, size_t* out_bytes);

/* Workspace (device scratch, 256-byte aligned) needed by llm42_verify_window for
 * any call of 1 .. max_seqs sequences, the given window and contexts
 * (seq_len + n_valid) up to max_context. */
llm42_status llm42_workspace_bytes(const llm42_model* model, int32_t max_seqs, int32_t window,
                                   int32_t max_context, size_t* out_bytes);

/* Verifier pass over a group of sequences [Sections 4.2, 4.3].
 *
 * Row (s, i), i < n_valid[s], is input token candidates[s][i] at absolute position
 * seq_lens[s] + i.  candidates[s][0] must be a consistent token and the first
 * seq_lens[s] cache entries of s must be consistent (the caller's precondition;
 * Section 4.2 requires the verifier's first input to come from a consistent state).
 * Effects, all on `hip_stream`:
 *   - cache slots seq_lens[s] .. seq_lens[s]+n_valid[s]-1 of every layer are
 *     overwritten with the verifier's K and V; no other slot is written and no
 *     slot at or beyond seq_lens[s]+n_valid[s] is ever read;
 *   - out_tokens[s][i] = arg-max (lowest index on ties) of the logits of row
 *     (s, i); -1 for padding rows i >= n_valid[s] and for every row of a sequence
 *     whose status is not LLM42_SEQ_OK (such a sequence is skipped entirely);
 *   - if n_dump > 0: out_logits[j][i][:] = fp32 logits of row (dump_seq_ids[j], i)
 *     (rows that are padding are left untouched).
 * max_context: host-known upper bound on seq_lens[s] + n_valid[s]; it sizes the
 * attention grid.  LLM42_ECAPACITY if it exceeds max_blocks_per_seq*16 or
 * cfg.max_position. */
llm42_status llm42_verify_window(
    const llm42_model*    model,
    const llm42_kv_cache* kv_cache,
    const int32_t*        seq_lens,      /* dev [num_seqs]                               */
    const int32_t*        candidates,    /* dev [num_seqs][window]                       */
    int32_t               window,        /* 1 .. LLM42_MAX_WINDOW                        */
    const int32_t*        n_valid,       /* dev [num_seqs] or NULL (= window everywhere) */
    int32_t               num_seqs,      /* >= 1, num_seqs * window <= LLM42_MAX_ROWS    */
    int32_t               max_context,
    int32_t*              out_tokens,    /* dev [num_seqs][window]                       */
    int32_t*              seq_status,    /* dev [num_seqs] or NULL                       */
    float*                out_logits,    /* dev [n_dump][window][vocab] or NULL          */
    const int32_t*        dump_seq_ids,  /* dev [n_dump] or NULL                         */
    int32_t               n_dump,
    void*                 workspace,     /* dev                                          */
    size_t                workspace_bytes,
    void*                 hip_stream);   /* hipStream_t; NULL = default stream           */

/* llm42_verify_window for callers that cannot allocate or pass device scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, effects and
 * results (bit for bit) as llm42_verify_window, without `workspace`: the pass runs in a scratch
 * area of LLM42_STATIC_SCRATCH_BYTES that is part of the library's device image (each GPU on which
 * a model was created holds one copy until the process ends; its device address is looked up once
 * per device in llm42_model_create).  The call allocates nothing and frees nothing.
 * LLM42_EWORKSPACE if the call needs more than the area holds (what it needs is
 * llm42_workspace_bytes of its own num_seqs, window and max_context); LLM42_EINVAL if the model's
 * device is not the current one.  All calls on one GPU share the one area, which keeps the
 * previous call's contents (every pass rewrites what it reads, nothing has to start at zero):
 * calls that overlap in time on the same GPU - other streams, other threads - race; order them. */
#define LLM42_STATIC_SCRATCH_BYTES (64u << 20)
llm42_status llm42_verify_window_static(
    const llm42_model* model, const llm42_kv_cache* kv_cache, const int32_t* seq_lens, const int32_t* candidates,
    int32_t window, const int32_t* n_valid, int32_t num_seqs, int32_t max_context, int32_t* out_tokens,
    int32_t* seq_status, float* out_logits, const int32_t* dump_seq_ids, int32_t n_dump, void* hip_stream);

/* Accept rule [Section 4.2].  For sequence s with n = n_valid[s] inputs:
 * m = number of leading candidates with candidates[s][i+1] == out_tokens[s][i],
 * i < n-1.  committed_counts[s] = m+1 (>= 1: forward progress); committed_tokens
 * [s][0..m] = out_tokens[s][0..m] (entries beyond are set to -1);
 * rolled_back_counts[s] = n-1-m; seq_lens[s] += m+1, which IS the KV truncation:
 * entries beyond the new length are dead.  A sequence with out_tokens[s][0] < 0
 * (skipped by the verifier) commits nothing: counts 0, seq_lens unchanged.
 * Integer work only. */
llm42_status llm42_commit_rollback(
    const int32_t* candidates,          /* dev [num_seqs][window]            */
    const int32_t* out_tokens,          /* dev [num_seqs][window]            */
    const int32_t* n_valid,             /* dev [num_seqs] or NULL (= window) */
    int32_t        num_seqs,
    int32_t        window,
    int32_t*       seq_lens,            /* dev [num_seqs], in/out            */
    int32_t*       committed_counts,    /* dev [num_seqs], out               */
    int32_t*       committed_tokens,    /* dev [num_seqs][window], out       */
    int32_t*       rolled_back_counts,  /* dev [num_seqs] or NULL, out       */
    void*          hip_stream);

/* Seeded stochastic sampling (SS 4.4 "Sampling": for temperature > 0 the logits are perturbed with
 * Gumbel noise generated by a seeded hash, so that the same input and seed always give the same token).
 * With temperature > 0 the token of a row is  argmax_v( logit_v / temperature + g_v ),  lowest index
 * on ties, where g_v = -log(-log(u_v)), u_v = (2 * (h >> 41) + 1) / 2^24 and
 * h = mix(mix(mix(seed ^ mix(request_id)) ^ position) ^ v);  mix is the output function of the
 * splitmix64 generator applied to its argument (add 0x9E3779B97F4A7C15; xor-shift 30, multiply
 * 0xBF58476D1CE4E5B9; xor-shift 27, multiply 0x94D049BB133111EB; xor-shift 31), position is the
 * row's absolute position in its sequence and request_id the caller's id of the sequence.
 * temperature == 0 (or a NULL llm42_sampling) is the greedy sampler.  out_logits, if asked for,
 * always receives the unperturbed logits. */
typedef struct {
  float          temperature;         /* >= 0                                             */
  uint64_t       seed;
  const int64_t* request_ids;         /* dev [num_seqs]; NULL: the index in the call      */
} llm42_sampling;

/* llm42_verify_window / llm42_decode_step with the sampler above in place of the arg-max. */
llm42_status llm42_verify_window_sampled(
    const llm42_model* model, const llm42_kv_cache* kv_cache, const int32_t* seq_lens, const int32_t* candidates,
    int32_t window, const int32_t* n_valid, int32_t num_seqs, int32_t max_context, int32_t* out_tokens,
    int32_t* seq_status, float* out_logits, const int32_t* dump_seq_ids, int32_t n_dump,
    void* workspace, size_t workspace_bytes, void* hip_stream, const llm42_sampling* sampling);
llm42_status llm42_decode_step_sampled(
    const llm42_model* model, const llm42_kv_cache* kv_cache, const int32_t* seq_lens, const int32_t* tokens,
    int32_t num_seqs, int32_t max_context, int32_t* out_tokens, int32_t* seq_status,
    void* workspace, size_t workspace_bytes, void* hip_stream, const llm42_sampling* sampling);

/* Fast path (SS 4.1: candidate tokens come from ordinary, high-throughput decoding whose reduction
 * order follows the batch): one greedy decoding step for num_seqs sequences.  tokens[s] is the input
 * token of sequence s at position seq_lens[s]; its K and V are written to that slot of the cache
 * (an unverified entry: the next llm42_verify_window over the position overwrites it) and
 * out_tokens[s] receives the arg-max token.  Same kernels as the verifier, but the split of the
 * residual projections follows the number of rows (two k-halves up to 16 rows, none beyond), so the
 * low bits of the logits - and now and then a token - depend on how many sequences are decoded
 * together.  That is what the verifier exists to repair.  dev [num_seqs] arrays; workspace as for
 * llm42_verify_window with window 1; errors and seq_status as there. */
llm42_status llm42_decode_step(
    const llm42_model* model, const llm42_kv_cache* kv_cache, const int32_t* seq_lens, const int32_t* tokens,
    int32_t num_seqs, int32_t max_context, int32_t* out_tokens, int32_t* seq_status,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Deterministic prefill (SS 4.1, use of observation O3: prefill is made deterministic by itself, without
 * a verifier; SS 4.2: the first output token T_0 comes from it.  The limitations paragraph that closes
 * SS 5 says the prototype cannot share prefix caches because its prefill and its decoding reduce
 * differently; here prefill IS the verifier run over the prompt, and the
 * verifier's result at a position depends on the tokens up to it only, never on how they were cut
 * into passes or batched, so a cached prefix can be shared).  For every sequence s the tokens
 * prompt_tokens[prompt_offsets[s] .. prompt_offsets[s+1]) are appended behind the seq_lens[s]
 * positions that its block table already holds (0 for a fresh sequence; the length of a shared or
 * previously cached prefix otherwise): the call runs ceil(max_prompt_len / chunk) verifier passes of
 * `chunk` rows per sequence, which write the prompt's K and V, and out_next_tokens[s] receives the
 * verifier's token after the last prompt token - the first consistent token T_0 of the decoding
 * loop, whose own K and V are not cached yet.  seq_lens is not modified; the consistent length after
 * the call is seq_lens[s] + the prompt's length.  A sequence with an empty prompt takes no part and
 * gets -1.  max_prompt_len (host) must be at least the longest prompt; max_context bounds
 * seq_lens[s] + prompt length.  seq_status (or NULL) receives the OR of the passes' status bits, a
 * prompt longer than max_prompt_len counting as LLM42_SEQ_BAD_LENGTH; a flagged sequence gets -1 and
 * its cache slots hold nothing usable.  sampling: NULL for the greedy sampler.
 * Workspace: llm42_prefill_workspace_bytes(model, num_seqs, chunk, max_context) bytes, 256-byte aligned.
 * Enqueues on hip_stream and returns; allocates nothing; reads no device memory on the host. */
llm42_status llm42_prefill_workspace_bytes(const llm42_model* model, int32_t max_seqs, int32_t chunk,
                                           int32_t max_context, size_t* out_bytes);
llm42_status llm42_prefill(
    const llm42_model*    model,
    const llm42_kv_cache* kv_cache,        /* the prompt's slots are written                */
    const int32_t*        seq_lens,        /* dev [num_seqs]: positions already cached      */
    const int32_t*        prompt_tokens,   /* dev: all prompts, one after the other         */
    const int32_t*        prompt_offsets,  /* dev [num_seqs + 1], ascending                 */
    int32_t               num_seqs,
    int32_t               max_prompt_len,  /* host: >= every prompt's length                */
    int32_t               chunk,           /* rows per sequence and pass, 1 .. LLM42_MAX_WINDOW */
    int32_t               max_context,
    int32_t*              out_next_tokens, /* dev [num_seqs]                                */
    int32_t*              seq_status,      /* dev [num_seqs] or NULL                        */
    void* workspace, size_t workspace_bytes, void* hip_stream,
    const llm42_sampling* sampling);       /* or NULL                                       */

/* Description of the last error on this thread (host string, never NULL). */
const char* llm42_last_error(void);

/* Library version and the reduction-schedule constants that define the bits of
 * every result (for logs; changing any of them changes the low bits of logits). */
const char* llm42_schedule_info(void);

#ifdef __cplusplus
}
#endif
#endif /* LLM42_H_ */
