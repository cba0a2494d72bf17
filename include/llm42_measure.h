/* llm42_measure.h -- measurement aids of the verifier library (bench.py and the
 * tests use them; no caller of the protocol needs them).  They are kept out of
 * llm42.h on purpose: nothing declared here can change the result of a call
 * declared there.
 */
#ifndef LLM42_MEASURE_H_
#define LLM42_MEASURE_H_

#include "llm42.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-launch timing (process-wide state, not thread safe; it times launches, it never changes a result).
 * While enabled, every kernel launch of class `kind` (LLM42_K_*, or -1 for all
 * classes) made by the hot calls is bracketed by HIP events recorded on the
 * call's own stream, up to max_launches launches (further ones go untimed).
 * llm42_profile_collect waits for the recorded events, writes the duration of each
 * bracketed launch in milliseconds (and its class) in launch order to HOST arrays of
 * `capacity` entries, stores the count in *n_out, and disables timing again.  Events
 * are created inside llm42_profile_enable, never inside a hot call. */
enum {
  LLM42_K_PREPARE = 0, LLM42_K_EMBED, LLM42_K_RMSNORM, LLM42_K_QKV, LLM42_K_ATTENTION, LLM42_K_O_PROJ,
  LLM42_K_GATE_UP, LLM42_K_DOWN, LLM42_K_LM_HEAD, LLM42_K_ARGMAX, LLM42_K_COMMIT, LLM42_K_COUNT
};
llm42_status llm42_profile_enable(int32_t kind, int32_t max_launches);
llm42_status llm42_profile_collect(float* ms_out, int32_t* kinds_out, int32_t capacity, int32_t* n_out);

/* The cost of the fixed reduction schedule [the paper prices its own batch-invariant mode in
 * SS 2.3 and SS 5.1].  Same arguments and effects as llm42_verify_window, but THIS call - and
 * no other: the mode is an argument of the pass, not a state of the library - lets the
 * batch decide where the schedule costs time, as an ordinary engine would: with more than 16 rows the
 * two residual projections are not split along k (one accumulator per element instead of the
 * scheduled partial sums), and an attention workgroup that owns a whole 2048-key super
 * accumulates straight through it instead of closing a partial every 256 keys.  Results stay
 * within rounding of llm42_verify_window's but are not bitwise independent of the batch.
 * It runs the same tile kernels as the verifier, so the difference it shows is a lower bound
 * on what an engine with freely chosen split-K and KV splits would gain. */
llm42_status llm42_measure_verify_window_batch_chosen(
    const llm42_model* model, const llm42_kv_cache* kv_cache, const int32_t* seq_lens, const int32_t* candidates,
    int32_t window, const int32_t* n_valid, int32_t num_seqs, int32_t max_context, int32_t* out_tokens,
    int32_t* seq_status, float* out_logits, const int32_t* dump_seq_ids, int32_t n_dump,
    void* workspace, size_t workspace_bytes, void* hip_stream);

/* How a call of this shape distributes its attention work (the distribution never changes a bit
 * of the result; tests use this to know which kernels a case exercised).  Writes five values to
 * the HOST array `out`:
 *   out[0]  keys per work item: 256 (one workgroup per chunk, all folds in the merge pass) or
 *           2048 (one per super, chunks folded in registers);
 *   out[1]  1 if every context fits one 2048-key unit and the attention kernel writes the
 *           output itself (no merge pass);
 *   out[2]  1 if the call may take whole sequences as work items - the device decides from the
 *           lengths whether they deal out evenly enough;
 *   out[3]  byte offset, in the call's workspace, of the int32 that the device sets to 1 when
 *           it did take whole sequences (valid after the call has run);
 *   out[4]  1 if the 8-wave streaming kernel runs (8 or more blocks of 16 query rows per
 *           sequence and kv head), 0 for the 4-wave kernel. */
llm42_status llm42_measure_attention_plan(const llm42_model* model, int32_t num_seqs, int32_t window,
                                          int32_t max_context, int64_t* out);

#ifdef __cplusplus
}
#endif
#endif /* LLM42_MEASURE_H_ */
