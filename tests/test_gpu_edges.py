"""GPU parity on edge cases of the small configuration, element by element against the checker:
the widest window (64 rows per sequence: the 8-wave attention stream and the mid-size tiled GEMM),
ragged n_valid, an empty prefix, a window of one row, and contexts that end just before, on and
just after the boundaries of the attention schedule (64-key steps, 256-key chunks)."""
import numpy as np
import pytest
import torch

from helpers import orc, wl, oracle_cfg, oracle_prefill
from gpu_helpers import (VerifierSession, assert_logits_close, oracle_kv_to_gpu, gpu_kv_tokens,
                         assert_tokens_match_where_decidable)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def tiny():
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, w, max_position=1024, device=DEV)
    yield shape, w, sess
    sess.close()


def _checker_state(shape, w, lens, window, seed):
    """Prompts of the given lengths prefilled by the checker; random candidate windows."""
    cfg = oracle_cfg(shape)
    rng = wl.rng_for(seed, 7)
    caches = []
    for n in lens:
        kv = orc.OracleKV(cfg, int(n) + window)
        if n > 0:
            oracle_prefill(cfg, w, kv, wl.random_tokens(rng, int(n), shape.vocab))
        caches.append(kv)
    cand = wl.random_tokens(rng, len(lens) * window, shape.vocab).reshape(len(lens), window).astype(np.int32)
    return cfg, caches, cand


def _run_and_compare(tiny, lens, window, n_valid, seed):
    shape, w, sess = tiny
    lens = np.asarray(lens, dtype=np.int32)
    cfg, caches, cand = _checker_state(shape, w, lens, window, seed)
    table, num_blocks = wl.make_block_table(wl.rng_for(seed, 8), lens + window, 16, spare_blocks=5)
    kv = sess.kv_cache(num_blocks)
    kv.fill_(float("nan"))                      # whatever is read without having been written shows up
    bt = torch.as_tensor(table, device=DEV)
    for s, okv in enumerate(caches):
        if lens[s] > 0:
            oracle_kv_to_gpu(kv, bt[s], okv, int(lens[s]))
    nv = None if n_valid is None else torch.as_tensor(np.asarray(n_valid, dtype=np.int32), device=DEV)
    dump = torch.arange(len(lens), dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, torch.as_tensor(lens, device=DEV), torch.as_tensor(cand, device=DEV),
                                      n_valid=nv, dump_seq_ids=dump)
    torch.cuda.synchronize()
    assert status.tolist() == [0] * len(lens)
    o_tokens, o_logits = orc.verify_window(cfg, w, caches, lens, cand, n_valid)
    out_c = out.cpu().numpy()
    for s in range(len(lens)):
        n = window if n_valid is None else int(n_valid[s])
        assert_logits_close(logits[s, :n], o_logits[s], f"L={int(lens[s])} n={n}")
        assert_tokens_match_where_decidable(out_c[s, :n], logits[s, :n], o_tokens[s], o_logits[s], f"seq {s}")
        assert (out_c[s, n:] == -1).all()       # padding rows carry no result
        # the window's K/V slots now hold the verifier's values, bf16 like the checker's cache
        k, v = gpu_kv_tokens(kv, bt[s], int(lens[s]) + n, shape.head_dim)
        ok, ov = caches[s].k[:, :int(lens[s]) + n].double(), caches[s].v[:, :int(lens[s]) + n].double()
        assert float((k - ok).abs().max()) <= 2e-2 and float((v - ov).abs().max()) <= 2e-2


def test_widest_window_ragged_rows_and_an_empty_prefix(tiny):
    # 3 x 64 = 192 rows: mid-size tiled GEMM; 2 q heads per kv head x 64 rows = 8 row blocks: attention stream
    _run_and_compare(tiny, lens=[0, 37, 255], window=64, n_valid=[64, 1, 33], seed=101)


def test_windows_beyond_64_rows_per_sequence(tiny):
    # the window ablation of the paper's section 5.3 goes up to 512 inputs per request
    _run_and_compare(tiny, lens=[0, 37, 100], window=160, n_valid=[160, 129, 65], seed=105)
    _run_and_compare(tiny, lens=[20], window=512, n_valid=[500], seed=106)


def test_window_of_one_row(tiny):
    _run_and_compare(tiny, lens=[1, 63, 64, 300], window=1, n_valid=None, seed=102)


def test_contexts_around_step_and_chunk_boundaries(tiny):
    _run_and_compare(tiny, lens=[56, 63, 64, 248, 255, 256, 257, 511, 512], window=8, n_valid=None, seed=103)


def test_lifting_the_schedule_changes_rounding_only(tiny):
    """llm42_measure_verify_window_batch_chosen (bench only) lets the batch choose the split of the residual
    projections: the logits move by rounding, nothing else; the mode belongs to that one call, so the
    verifier's own calls before and after it give the same bits."""
    from paper_2601_17768_amd import binding as B
    shape, w, sess = tiny
    rng = wl.rng_for(104, 1)
    lens = np.array([40, 90, 130], dtype=np.int32)
    window = 64                                  # 192 rows: above the 64-row limit of the small-batch kernels
    table, num_blocks = wl.make_block_table(rng, lens + window, 16, spare_blocks=2)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(5))
    bt = torch.as_tensor(table, device=DEV)
    cand = torch.as_tensor(wl.random_tokens(rng, 3 * window, shape.vocab).reshape(3, window).astype(np.int32), device=DEV)
    dump = torch.arange(3, dtype=torch.int32, device=DEV)
    sl = torch.as_tensor(lens, device=DEV)
    max_context = bt.shape[1] * 16
    _, _, fixed = sess.verify(kv, bt, sl, cand, dump_seq_ids=dump)
    fixed = fixed.clone()
    free = torch.zeros_like(fixed)
    out = torch.empty((3, window), dtype=torch.int32, device=DEV)
    B.llm42_verify_window(sess.model, kv, num_blocks, bt, sl, cand, window, None, max_context, out,
                          sess.workspace(3, window, max_context), None, free, dump, batch_chosen=True)
    _, _, again = sess.verify(kv, bt, sl, cand, dump_seq_ids=dump)
    torch.cuda.synchronize()
    assert torch.equal(again, fixed)
    assert not torch.equal(free, fixed)          # a different reduction order does show in the last bits
    assert float((free - fixed).abs().max()) < 2e-2   # the logit tolerance; measured 4e-3 (bf16 rounding points amplify last-bit differences)


def test_one_workspace_serves_every_smaller_call(tiny):
    """llm42_workspace_bytes(max_seqs, ...) is enough for every call of 1 .. max_seqs sequences, although a call
    of fewer sequences may split its attention work finer (per 256-key chunk instead of per 2048-key super) and
    then needs more partial slots per sequence."""
    from paper_2601_17768_amd import binding as B
    shape, w, sess = tiny
    window, max_seqs, max_context = 16, 110, 512
    rng = wl.rng_for(105, 1)
    ws = torch.empty(B.llm42_workspace_bytes(sess.model, max_seqs, window, max_context), dtype=torch.uint8, device=DEV)
    modes = set()
    lens = wl.uniform_lengths(rng, max_seqs, 1, max_context - window)
    table, num_blocks = wl.make_block_table(rng, lens + window, 16, max_blocks_per_seq=max_context // 16, spare_blocks=2)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(6))
    bt = torch.as_tensor(table, device=DEV)
    cand = torch.as_tensor(wl.random_tokens(rng, max_seqs * window, shape.vocab).reshape(max_seqs, window).astype(np.int32), device=DEV)
    sl = torch.as_tensor(lens, device=DEV)
    for n in range(1, max_seqs + 1):
        assert B.llm42_workspace_bytes(sess.model, n, window, max_context) <= ws.numel()
        plan = B.llm42_measure_attention_plan(sess.model, n, window, max_context)
        modes.add((plan["item_keys"], plan["direct"]))
        out = torch.empty((n, window), dtype=torch.int32, device=DEV)
        B.llm42_verify_window(sess.model, kv, num_blocks, bt[:n].contiguous(), sl[:n].contiguous(), cand[:n].contiguous(),
                              window, None, max_context, out, ws)
    torch.cuda.synchronize()
    assert int(out.min()) >= 0
    assert modes == {(256, False), (2048, True)}      # both work splits were crossed
