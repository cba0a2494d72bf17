"""Full 8B shape (32 layers, d 4096, 32 q / 8 kv heads of 128, FFN 14336, vocab
128256, random-init): parity with the stored float64 checker results of the
single-sequence configuration, the batch-invariance stress, and the grouped
32-sequence and 128-sequence configurations checked through properties that hold at any size."""
import json
import os

import numpy as np
import pytest
import torch

from helpers import orc, wl
from helpers import oracle_cfg
from gpu_helpers import (VerifierSession, gpu_kv_tokens, assert_logits_within_noise, checker_noise,
                         assert_tokens_match_where_decidable)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "c2_llama8b_window32.json")
MAX_POS = 8320


@pytest.fixture(scope="module")
def big():
    shape = wl.LLAMA_8B
    w = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, w, max_position=MAX_POS, device=DEV)
    yield shape, sess, w
    sess.close()


@pytest.mark.timeout(900)
def test_c2_single_sequence_against_stored_checker_results(big):
    """Inputs are regenerated from the seed exactly as tests/golden/make_c2_golden.py does;
    the prompt's KV comes from the library's own prefill, so the comparison covers
    prefill + verify end to end."""
    shape, sess, w = big
    gold = json.load(open(GOLDEN))
    window, plen = gold["window"], gold["prompt_len"]
    prompt = wl.random_tokens(wl.rng_for(gold["seed"], 2, 0), plen, shape.vocab)
    cols = torch.as_tensor(gold["columns"])
    table, num_blocks = wl.make_block_table(wl.rng_for(7), [plen + window], 16, spare_blocks=3)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks, fill=float("nan"))
    first = sess.prefill(kv, bt, [prompt], window=32)
    cand = torch.as_tensor(np.array([gold["candidates"]], dtype=np.int32), device=DEV)
    seq_lens = torch.tensor([plen], dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, seq_lens, cand, dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV))
    counts, ctoks, rolled = sess.commit(cand, out, seq_lens)
    torch.cuda.synchronize()
    assert int(status[0]) == 0
    lg = logits[0].cpu().double()
    # sampled columns + the checker's top-2 columns of every row
    ref_cols = torch.tensor(gold["logits_at_columns"], dtype=torch.float64)
    top_ids = torch.tensor(gold["top2_ids"])
    ref_top = torch.tensor(gold["top2_values"], dtype=torch.float64)
    got = torch.cat([lg[:, cols], torch.gather(lg, 1, top_ids)], dim=1)
    ref = torch.cat([ref_cols, ref_top], dim=1)
    err, rms = assert_logits_within_noise(got, ref, gold["self_noise"]["model_rms"], gold["self_noise"]["model_max"],
                                          "c2 sampled logits")
    assert abs(float(lg.std()) - gold["logit_std"]) < 0.01
    # tokens: decidable where the checker's margin exceeds twice the row's error bound
    bound = max(err, float((got - ref).abs().max()))
    margin = ref_top[:, 0] - ref_top[:, 1]
    exempt = 0
    for i in range(window):
        if float(margin[i]) > 2 * bound:
            assert int(out[0, i]) == gold["out_tokens"][i], i
        else:
            exempt += 1
    print(f"c2: logit error max {err:.3e} rms {rms:.3e}; rows exempt from the token check: {exempt} of {window}")
    if float(margin.min()) > 2 * bound:
        assert int(first[0]) == gold["first_token"]
        assert int(counts[0]) == gold["committed"] and int(rolled[0]) == gold["rolled_back"]
        assert ctoks[0, :gold["committed"]].tolist() == gold["committed_tokens"]
        assert int(seq_lens[0]) == plen + gold["committed"]
    c, t, r = orc.commit_rollback(gold["candidates"], out[0].tolist(), window)
    assert (int(counts[0]), int(rolled[0])) == (c, r) and int(seq_lens[0]) == plen + c
    # K/V written by the verifier for the window
    k, v = gpu_kv_tokens(kv, bt[0], plen + window, shape.head_dim)
    for li, layer in enumerate(gold["kv_samples"]["layers"]):
        gk = torch.tensor(gold["kv_samples"]["k"][li], dtype=torch.float64)      # [window][2 heads][8]
        gv = torch.tensor(gold["kv_samples"]["v"][li], dtype=torch.float64)
        mk = k[layer, plen:plen + window][:, [0, 7], :8]
        mv = v[layer, plen:plen + window][:, [0, 7], :8]
        assert float((mk - gk).abs().max()) < 0.05 * max(1.0, float(gk.abs().max())), layer
        assert float((mv - gv).abs().max()) < 0.05 * max(1.0, float(gv.abs().max())), layer


def _compare_sequences_with_checker(shape, w, kv, bt, ctx, window, cand_host, out, logits, sample, what):
    """Sampled sequences of a large call against the float64 checker run on the very KV bytes the call read
    (read back from the paged cache): logits within the checker's own noise on the same inputs, tokens where the
    checker's margin decides, and the K/V the call wrote for the window."""
    cfg = oracle_cfg(shape)
    for j, s in enumerate(sample):
        L = int(ctx[s])
        k, v = gpu_kv_tokens(kv, bt[s], L + window, shape.head_dim)          # [layers, L + window, kv heads, head_dim]
        okv = orc.OracleKV(cfg, L + window)
        okv.k[:, :L] = k[:, :L]
        okv.v[:, :L] = v[:, :L]
        ref = orc.forward_window(cfg, w, okv, L, cand_host[s])
        noise = checker_noise(cfg, w, k, v, L, cand_host[s], ref)
        assert_logits_within_noise(logits[j], ref, float((noise * noise).mean().sqrt()), float(noise.max()),
                                   f"{what} sequence {s} (context {L})")
        exempt = assert_tokens_match_where_decidable(out[s].cpu(), logits[j], orc.greedy_argmax(ref), ref, f"{what} seq {s}")
        print(f"{what} sequence {s}: rows exempt from the token check {exempt} of {window}", flush=True)
        for name, got, want in (("K", k[:, L:], okv.k[:, L:L + window]), ("V", v[:, L:], okv.v[:, L:L + window])):
            d = (got - want).abs()
            assert float(d.max()) < 0.05 * max(1.0, float(want.abs().max())), (what, s, name, float(d.max()))


@pytest.mark.timeout(1500)
def test_c4_batch_invariance_stress(big):
    """One fixed target (context 1024, window 32) verified inside batches of 1, 2, 7, 32, 128
    and 256 other sequences (contexts uniform 64-4096, KV filled with seeded noise) at the
    first, middle and last slot, 5 runs each: logits, tokens and written KV are bitwise identical."""
    shape, sess, w = big
    window, ctx = 32, 1024
    rng = wl.rng_for(42, 4)
    prompt = wl.random_tokens(rng, ctx, shape.vocab)
    target_win = wl.random_tokens(rng, window, shape.vocab)
    ref = None
    for others in (0, 1, 2, 7, 32, 128, 256):
        comp_ctx = wl.uniform_lengths(rng, others, 64, 4096)
        for slot in sorted({0, others // 2, others}):
            lens = np.concatenate([comp_ctx[:slot], [ctx], comp_ctx[slot:]]).astype(np.int32)
            table, num_blocks = wl.make_block_table(rng, lens + window, 16, spare_blocks=2)
            bt = torch.as_tensor(table, device=DEV)
            kv = sess.kv_cache(num_blocks)
            kv.normal_(generator=torch.Generator(device=DEV).manual_seed(1000 + others))
            sess.prefill(kv, bt[slot:slot + 1].contiguous(), [prompt], window=64)
            cand = torch.as_tensor(wl.random_tokens(rng, (others + 1) * window, shape.vocab).reshape(-1, window),
                                   device=DEV).clone()
            cand[slot] = torch.as_tensor(target_win, device=DEV)
            seq_lens = torch.as_tensor(lens, device=DEV)
            dump = torch.tensor([slot], dtype=torch.int32, device=DEV)
            for rep in range(5 if others else 1):
                out, status, logits = sess.verify(kv, bt, seq_lens, cand, dump_seq_ids=dump,
                                                  max_context=int(lens.max()) + window)
                torch.cuda.synchronize()
                assert int(status.max()) == 0
                k, v = gpu_kv_tokens(kv, bt[slot], ctx + window, shape.head_dim)
                got = (logits[0].clone(), out[slot].clone(), k[:, ctx:], v[:, ctx:])
                if ref is None:
                    ref = got
                    assert torch.isfinite(ref[0]).all()
                else:
                    for a, b in zip(ref, got):
                        assert torch.equal(a, b), (others, slot, rep)
            del kv
            print(f"c4: {others} others, slot {slot}: identical", flush=True)


@pytest.mark.timeout(900)
def test_c3_grouped_sequences_properties(big):
    """32 sequences, prompt ~ lognormal(6.0, 1.0) in [16, 4096] plus generated ~ lognormal(5.3, 0.9)
    in [1, 2048] tokens of context, block size 16 with scattered blocks, window 64, 1 % replaced.
    Properties that hold at any size: each sampled sequence verified alone gives
    bitwise the same logits and tokens; the commit rule is exact on the library's own tokens;
    committed + rolled back = window; candidates equal to the verifier's own chain commit fully.
    Then two sampled sequences are compared with the checker run on the KV the call read."""
    shape, sess, w = big
    window, n_seq = 64, 32
    rng = wl.rng_for(42, 3)
    ctx = np.minimum(wl.lognormal_lengths(rng, n_seq, 6.0, 1.0, 16, 4096) +
                     wl.lognormal_lengths(rng, n_seq, 5.3, 0.9, 1, 2048), MAX_POS - window).astype(np.int32)
    table, num_blocks = wl.make_block_table(rng, ctx + window, 16, spare_blocks=4)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(3))
    seq_lens = torch.as_tensor(ctx, device=DEV)
    first = torch.as_tensor(wl.random_tokens(rng, n_seq, shape.vocab), device=DEV)
    # greedy chain by iterating the verifier to its fixed point
    cand = torch.zeros((n_seq, window), dtype=torch.int32, device=DEV)
    cand[:, 0] = first
    for it in range(window):
        out, status, _ = sess.verify(kv, bt, seq_lens, cand, max_context=int(ctx.max()) + window)
        new = cand.clone()
        new[:, 1:] = out[:, :-1]
        if torch.equal(new, cand):
            break
        cand = new
    assert int(status.max()) == 0
    lens = seq_lens.clone()
    counts, _, rolled = sess.commit(cand, out, lens)
    assert counts.tolist() == [window] * n_seq and rolled.tolist() == [0] * n_seq
    replaced = torch.as_tensor(wl.replace_candidates(rng, cand.cpu().numpy(), 0.01, shape.vocab), device=DEV)
    sample = [0, 13, 31]
    dump = torch.tensor(sample, dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, seq_lens, replaced, dump_seq_ids=dump, max_context=int(ctx.max()) + window)
    lens = seq_lens.clone()
    counts, ctoks, rolled = sess.commit(replaced, out, lens)
    torch.cuda.synchronize()
    rep_host, out_host = replaced.cpu().numpy(), out.cpu().numpy()
    for s in range(n_seq):
        c, t, r = orc.commit_rollback(rep_host[s], out_host[s], window)
        assert (int(counts[s]), int(rolled[s])) == (c, r) and c + r == window and int(lens[s]) == ctx[s] + c
        assert ctoks[s, :c].tolist() == t
    assert 1 <= int(counts.min()) and int(counts.sum()) < n_seq * window      # some rollbacks happened
    for j, s in enumerate(sample):
        o1, st1, lg1 = sess.verify(kv, bt[s:s + 1].contiguous(), seq_lens[s:s + 1].contiguous(),
                                   replaced[s:s + 1].contiguous(), dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV),
                                   max_context=int(ctx[s]) + window)
        torch.cuda.synchronize()
        assert torch.equal(lg1[0], logits[j]) and torch.equal(o1[0], out[s])
    # and two of them against the checker itself
    _compare_sequences_with_checker(shape, w, kv, bt, ctx, window, rep_host, out, logits, sample[:2], "c3")


@pytest.mark.timeout(900)
def test_c5_many_long_sequences_properties(big):
    """128 sequences with contexts uniform in [1024, 8192], window 32 (4096 rows per pass, about 75 GB of
    KV: the configuration the bench line times).  The
    commit rule is exact on the library's own tokens, sampled sequences verified alone give
    bitwise the same logits, tokens and written K/V as inside the batch, and two of them are compared with
    the checker run on the KV the call read."""
    shape, sess, w = big
    window, n_seq = 32, 128
    rng = wl.rng_for(42, 5)
    ctx = wl.uniform_lengths(rng, n_seq, 1024, 8192)
    table, num_blocks = wl.make_block_table(rng, ctx + window, 16, spare_blocks=8)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(5))
    seq_lens = torch.as_tensor(ctx, device=DEV)
    cand = torch.as_tensor(wl.random_tokens(rng, n_seq * window, shape.vocab).reshape(n_seq, window).astype(np.int32),
                           device=DEV)
    max_context = int(ctx.max()) + window
    # one pass makes the candidates after the first input the verifier's own where they can be: some windows then match for a while
    out, status, _ = sess.verify(kv, bt, seq_lens, cand, max_context=max_context)
    cand[:, 1:4] = out[:, 0:3]
    sample = [0, 57, 127]
    dump = torch.tensor(sample, dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, seq_lens, cand, dump_seq_ids=dump, max_context=max_context)
    lens = seq_lens.clone()
    counts, ctoks, rolled = sess.commit(cand, out, lens)
    torch.cuda.synchronize()
    assert int(status.max()) == 0 and torch.isfinite(logits).all()
    cand_host, out_host = cand.cpu().numpy(), out.cpu().numpy()
    for s in range(n_seq):
        c, t, r = orc.commit_rollback(cand_host[s], out_host[s], window)
        assert (int(counts[s]), int(rolled[s])) == (c, r) and c + r == window and int(lens[s]) == ctx[s] + c
        assert ctoks[s, :c].tolist() == t
    assert int(counts.max()) >= 2                         # the first candidate, at least, was reproduced somewhere
    batch_kv = [gpu_kv_tokens(kv, bt[s], int(ctx[s]) + window, shape.head_dim) for s in sample]
    for j, s in enumerate(sample):
        o1, st1, lg1 = sess.verify(kv, bt[s:s + 1].contiguous(), seq_lens[s:s + 1].contiguous(), cand[s:s + 1].contiguous(),
                                   dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV),
                                   max_context=int(ctx[s]) + window)
        torch.cuda.synchronize()
        assert torch.equal(lg1[0], logits[j]) and torch.equal(o1[0], out[s]), s
        k, v = gpu_kv_tokens(kv, bt[s], int(ctx[s]) + window, shape.head_dim)
        assert torch.equal(k[:, ctx[s]:], batch_kv[j][0][:, ctx[s]:]) and torch.equal(v[:, ctx[s]:], batch_kv[j][1][:, ctx[s]:])
    del batch_kv
    # and two of them against the checker itself (whole-sequence attention items at head_dim 128, the tiled GEMMs at 4096 rows)
    _compare_sequences_with_checker(shape, w, kv, bt, ctx, window, cand_host, out, logits, sample[:2], "c5")
