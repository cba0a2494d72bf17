"""Every way the attention work of a call can be distributed, checked against the CPU checker
(element by element, spec tolerance) on contexts that reach past one, two and three
2048-key units: one workgroup per 256-key chunk (4-wave and 8-wave streaming kernels, all folds in
the merge pass), one per 2048-key super (chunks folded in registers, supers in the merge pass),
the attention kernel writing the output itself (contexts within one unit), and whole sequences
as work items (supers folded in registers too).  The distribution never changes a bit, so
the same target must also give the same bits in every company."""
import numpy as np
import pytest
import torch

from helpers import orc, wl, oracle_cfg
from gpu_helpers import (VerifierSession, assert_logits_close, assert_tokens_match_where_decidable, oracle_kv_to_gpu,
                         gpu_kv_tokens)
from paper_2601_17768_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOTAL = 6200 + 64


@pytest.fixture(scope="module")
def env():
    """One long token sequence prefilled by the checker: every context used below is a prefix of it."""
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    cfg = oracle_cfg(shape)
    tokens = wl.random_tokens(wl.rng_for(42, 61), TOTAL, shape.vocab)
    okv = orc.OracleKV(cfg, TOTAL)
    orc.forward_window(cfg, w, okv, 0, tokens)
    sess = VerifierSession(shape, w, max_position=6400, device=DEV)
    yield shape, w, cfg, tokens, okv, sess
    sess.close()


def _run(env, L, window, companions, slot, expect, seed):
    """Verify tokens[L : L + window] behind the checker's prefix, among `companions` (contexts, KV = seeded
    noise).  expect: item_keys / direct / streaming / sequences as the plan must report them."""
    shape, w, cfg, tokens, okv, sess = env
    rng = wl.rng_for(42, seed)
    lens = np.concatenate([companions[:slot], [L], companions[slot:]]).astype(np.int32)
    n_seq = len(lens)
    table, num_blocks = wl.make_block_table(rng, lens + window, 16, spare_blocks=3)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(seed))
    oracle_kv_to_gpu(kv, bt[slot], okv, L)
    cand = wl.random_tokens(rng, n_seq * window, shape.vocab).reshape(n_seq, window).astype(np.int32)
    cand[slot] = tokens[L:L + window]
    max_context = int(lens.max()) + window
    plan = B.llm42_measure_attention_plan(sess.model, n_seq, window, max_context)
    assert plan["item_keys"] == expect["item_keys"] and plan["direct"] == expect["direct"], plan
    assert plan["streaming"] == expect["streaming"] and plan["may_take_sequences"] == expect["sequences"], plan
    d = lambda a: torch.as_tensor(a, device=DEV)
    out, status, logits = sess.verify(kv, bt, d(lens), d(cand), dump_seq_ids=torch.tensor([slot], dtype=torch.int32, device=DEV),
                                      max_context=max_context)
    torch.cuda.synchronize()
    assert int(status.max()) == 0
    if expect["sequences"]:      # the device took whole sequences (the lengths of this call deal out evenly)
        flag = sess.workspace(n_seq, window, max_context)[plan["sequences_flag_offset"]:plan["sequences_flag_offset"] + 4]
        assert int(flag.view(torch.int32)[0]) == 1
    ref = orc.forward_window(cfg, w, okv, L, tokens[L:L + window])
    what = f"context {L} window {window} among {n_seq - 1} ({expect})"
    assert_logits_close(logits[0], ref, what)
    exempt = assert_tokens_match_where_decidable(out[slot].cpu(), logits[0], orc.greedy_argmax(ref), ref, what)
    assert exempt <= window // 4
    gk, gv = gpu_kv_tokens(kv, bt[slot], L + window, shape.head_dim)
    assert float((gk[:, L:] - okv.k[:, L:L + window]).abs().max()) < 2e-2
    assert float((gv[:, L:] - okv.v[:, L:L + window]).abs().max()) < 2e-2
    return logits[0].cpu()


CHUNK4 = dict(item_keys=256, direct=False, streaming=False, sequences=False)
CHUNK8 = dict(item_keys=256, direct=False, streaming=True, sequences=False)
SUPER4 = dict(item_keys=2048, direct=False, streaming=False, sequences=False)
SUPER8 = dict(item_keys=2048, direct=False, streaming=True, sequences=False)
DIRECT4 = dict(item_keys=2048, direct=True, streaming=False, sequences=False)
DIRECT8 = dict(item_keys=2048, direct=True, streaming=True, sequences=False)
SEQS = dict(item_keys=2048, direct=False, streaming=True, sequences=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("L", [2040, 2047, 2060, 4100, 6200])
def test_contexts_past_one_unit_in_every_distribution(env, L):
    rng = wl.rng_for(42, 62, L)
    none = np.zeros(0, dtype=np.int32)
    some = wl.uniform_lengths(rng, 100, 100, L)              # 101 sequences: one workgroup per super
    even = wl.uniform_lengths(rng, 255, L - 100, L)          # 256 sequences of about the same length: whole sequences
    # (window 8 behind 2040 keys ends exactly at the first unit's last key: such a call needs no merge pass)
    got8 = [_run(env, L, 8, none, 0, CHUNK4, 1), _run(env, L, 8, some, 17, DIRECT4 if L + 8 <= 2048 else SUPER4, 2)]
    got64 = [_run(env, L, 64, none, 0, CHUNK8, 3), _run(env, L, 64, some, 100, SUPER8, 4),
             _run(env, L, 64, even, 100, SEQS, 5)]
    for g in got8[1:]:
        assert torch.equal(g, got8[0])
    for g in got64[1:]:
        assert torch.equal(g, got64[0])
    assert torch.equal(got8[0], got64[0][:8])                # and the split into windows does not matter either


@pytest.mark.timeout(600)
def test_contexts_within_one_unit_without_a_merge_pass(env):
    L = 1970
    rng = wl.rng_for(42, 63)
    many = wl.uniform_lengths(rng, 63, 50, 1980)             # 64 sequences, every context within 2048 keys
    a = _run(env, L, 8, many, 40, DIRECT4, 6)
    b = _run(env, L, 64, many, 0, DIRECT8, 7)
    c = _run(env, L, 64, np.zeros(0, dtype=np.int32), 0, CHUNK8, 8)
    assert torch.equal(b, c) and torch.equal(a, b[:8])
