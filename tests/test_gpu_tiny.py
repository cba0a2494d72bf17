"""GPU parity on the small configuration (2 layers, d 256, 4 q / 2 kv heads of 64,
FFN 688, vocab 1024; 4 sequences, prompts of 16-64 tokens, window 8, 10 % of the
candidates replaced): the library is compared element by element with the checker."""
import numpy as np
import pytest
import torch

from helpers import orc, wl
from gpu_helpers import (Scenario, VerifierSession, assert_logits_close, oracle_kv_to_gpu, gpu_kv_tokens,
                         assert_tokens_match_where_decidable, ABS_TOL)
from paper_2601_17768_amd import kv_layout

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def tiny():
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, w, max_position=512, device=DEV)
    yield shape, w, sess
    sess.close()


@pytest.fixture(scope="module")
def scenario(tiny):
    shape, w, _ = tiny
    rng = wl.rng_for(42, 1)
    lens = wl.uniform_lengths(rng, 4, 16, 64)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in lens]
    return Scenario(shape, w, prompts, window=8, rate=0.10, seed=42)


def _setup_gpu(sess, sc, rng_stream=5, spare=3):
    table, num_blocks = wl.make_block_table(wl.rng_for(42, rng_stream), sc.lens + sc.window, 16, spare_blocks=spare)
    kv = sess.kv_cache(num_blocks)
    bt = torch.as_tensor(table, device=DEV)
    for s, okv in enumerate(sc.okv):
        oracle_kv_to_gpu(kv, bt[s], okv, int(sc.lens[s]))
    return kv, bt


def test_config1_logits_tokens_kv_and_commit(tiny, scenario):
    shape, w, sess = tiny
    sc = scenario
    kv, bt = _setup_gpu(sess, sc)
    seq_lens = torch.as_tensor(sc.lens, device=DEV)
    cand = torch.as_tensor(sc.candidates, device=DEV)
    dump = torch.arange(4, dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, seq_lens, cand, dump_seq_ids=dump)
    torch.cuda.synchronize()
    assert status.tolist() == [0, 0, 0, 0]
    o_tokens, o_logits = sc.oracle_verify()
    out_c = out.cpu().numpy()
    worst = 0.0
    for s in range(4):
        worst = max(worst, assert_logits_close(logits[s], o_logits[s], f"seq {s}")[0])
        assert_tokens_match_where_decidable(out_c[s], logits[s], o_tokens[s], o_logits[s], f"seq {s}")
        # the window's K/V now hold the verifier's values: compare with the checker's cache
        L, n = int(sc.lens[s]), sc.window
        gk, gv = gpu_kv_tokens(kv, bt[s], L + n, shape.head_dim)
        assert torch.equal(gk[:, :L], sc.okv[s].k[:, :L]) and torch.equal(gv[:, :L], sc.okv[s].v[:, :L])
        assert float((gk[:, L:] - sc.okv[s].k[:, L:L + n]).abs().max()) < 2e-2
        assert float((gv[:, L:] - sc.okv[s].v[:, L:L + n]).abs().max()) < 2e-2
    print(f"config 1: worst logit error {worst:.3e}")
    # commit / rollback: exact against the checker's rule applied to the GPU's own tokens,
    # and against the checker's tokens wherever the margins allow
    counts, toks, rolled = sess.commit(cand, out, seq_lens)
    torch.cuda.synchronize()
    for s in range(4):
        c, t, r = orc.commit_rollback(sc.candidates[s], out_c[s], sc.window)
        assert int(counts[s]) == c and int(rolled[s]) == r
        assert toks[s].tolist() == t + [-1] * (sc.window - c)
        assert int(seq_lens[s]) == int(sc.lens[s]) + c
        margin_ok = bool((orc.top2_margin(o_logits[s]) > 2 * ABS_TOL).all())
        if margin_ok:
            assert (c, t, r) == orc.commit_rollback(sc.candidates[s], o_tokens[s], sc.window)


def test_gpu_prefill_matches_checker_cache(tiny, scenario):
    """Teacher-forced prefill through the library reproduces the checker's cache and first token."""
    shape, w, sess = tiny
    sc = scenario
    table, num_blocks = wl.make_block_table(wl.rng_for(42, 6), sc.lens + sc.window, 16, spare_blocks=2)
    kv = sess.kv_cache(num_blocks, fill=float("nan"))
    bt = torch.as_tensor(table, device=DEV)
    first = sess.prefill(kv, bt, sc.prompts, window=8)
    torch.cuda.synchronize()
    for s in range(4):
        L = int(sc.lens[s])
        gk, gv = gpu_kv_tokens(kv, bt[s], L, shape.head_dim)
        assert float((gk - sc.okv[s].k[:, :L]).abs().max()) < 2e-2
        assert float((gv - sc.okv[s].v[:, :L]).abs().max()) < 2e-2
    assert first.tolist() == sc.first


def test_commit_kernel_exact_on_random_integers(tiny):
    _, _, sess = tiny
    rng = np.random.default_rng(3)
    for window in (1, 4, 8, 33, 64):
        B = 37
        x = rng.integers(0, 3, size=(B, window)).astype(np.int32)
        y = rng.integers(0, 3, size=(B, window)).astype(np.int32)
        nv = rng.integers(1, window + 1, size=B).astype(np.int32)
        y[5, 0] = -1                                    # a sequence the verifier skipped
        lens = rng.integers(0, 1000, size=B).astype(np.int32)
        d = lambda a: torch.as_tensor(a, device=DEV)
        seq_lens = d(lens.copy())
        counts, toks, rolled = sess.commit(d(x), d(y), seq_lens, d(nv))
        torch.cuda.synchronize()
        for s in range(B):
            if s == 5:
                assert int(counts[s]) == 0 and int(rolled[s]) == 0 and int(seq_lens[s]) == lens[s]
                continue
            c, t, r = orc.commit_rollback(x[s], y[s], int(nv[s]))
            assert (int(counts[s]), int(rolled[s])) == (c, r)
            assert toks[s].tolist() == t + [-1] * (window - c)
            assert int(seq_lens[s]) == lens[s] + c
