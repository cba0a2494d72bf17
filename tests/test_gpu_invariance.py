"""The determinism invariant (paper Sections 3 and 4.1): the verifier's logits for
a sequence are bitwise identical whatever the batch size, the batch composition,
the slot in the batch, the physical KV blocks, the split of the positions into
windows, stale data beyond the committed length, and across repeated runs."""
import numpy as np
import pytest
import torch

from helpers import orc, wl, oracle_cfg
from gpu_helpers import VerifierSession, assert_logits_close, gpu_kv_tokens
from paper_2601_17768_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def env():
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, w, max_position=2304, device=DEV)
    yield shape, w, sess
    sess.close()


def _batch(sess, shape, prompts, windows_tokens, window, slot_of_target, seed, kv_fill=0.0, n_valid=None):
    """Prefill `prompts` through the library, then verify one window per sequence.
    Returns logits of the sequence in `slot_of_target`, its window K/V and out tokens."""
    lens = np.array([len(p) for p in prompts], dtype=np.int32)
    table, num_blocks = wl.make_block_table(wl.rng_for(seed), lens + window, 16, spare_blocks=4)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks, fill=kv_fill)
    sess.prefill(kv, bt, prompts, window=16)
    seq_lens = torch.as_tensor(lens, device=DEV)
    cand = torch.as_tensor(np.stack(windows_tokens).astype(np.int32), device=DEV)
    dump = torch.tensor([slot_of_target], dtype=torch.int32, device=DEV)
    nv = None if n_valid is None else torch.as_tensor(np.asarray(n_valid, dtype=np.int32), device=DEV)
    out, status, logits = sess.verify(kv, bt, seq_lens, cand, n_valid=nv, dump_seq_ids=dump)
    torch.cuda.synchronize()
    assert int(status.max()) == 0
    L = int(lens[slot_of_target])
    k, v = gpu_kv_tokens(kv, bt[slot_of_target], L + window, shape.head_dim)
    return logits[0].cpu(), k[:, L:], v[:, L:], out[slot_of_target].cpu()


def test_batch_size_position_and_repeat_invariance(env):
    shape, w, sess = env
    window = 8
    rng = wl.rng_for(42, 4)
    target_prompt = wl.random_tokens(rng, 100, shape.vocab)
    target_window = wl.random_tokens(rng, window, shape.vocab)
    ref = _batch(sess, shape, [target_prompt], [target_window], window, 0, seed=1)
    checked = 0
    for others in (1, 2, 7, 12, 24, 32, 63, 90, 127):      # 16 .. 1024 rows: every GEMM kernel variant is crossed
        comp_lens = wl.uniform_lengths(rng, others, 8, 200)
        comp = [wl.random_tokens(rng, int(n), shape.vocab) for n in comp_lens]
        comp_win = [wl.random_tokens(rng, window, shape.vocab) for _ in range(others)]
        for slot in sorted({0, others // 2, others}):
            prompts = comp[:slot] + [target_prompt] + comp[slot:]
            wins = comp_win[:slot] + [target_window] + comp_win[slot:]
            for rep in range(2):
                got = _batch(sess, shape, prompts, wins, window, slot, seed=100 * others + slot + rep)
                for a, b in zip(ref, got):
                    assert torch.equal(a, b), (others, slot, rep)
                checked += 1
    assert checked == 9 * 3 * 2 - 2     # others=1 has two distinct slots only


def test_split_of_positions_into_windows_does_not_matter(env):
    """Prefix purity: logits at a position do not depend on the window it is verified in."""
    shape, w, sess = env
    rng = wl.rng_for(42, 5)
    prompt = wl.random_tokens(rng, 57, shape.vocab)
    tokens = wl.random_tokens(rng, 24, shape.vocab)
    table, num_blocks = wl.make_block_table(rng, [57 + 24], 16, spare_blocks=1)
    bt = torch.as_tensor(table, device=DEV)
    dump = torch.zeros(1, dtype=torch.int32, device=DEV)

    def run(cuts, window):
        kv = sess.kv_cache(num_blocks, fill=float("nan"))
        sess.prefill(kv, bt, [prompt], window=32)
        rows, at = [], 0
        for n in cuts:
            cand = np.zeros((1, window), dtype=np.int32)
            cand[0, :n] = tokens[at:at + n]
            _, status, logits = sess.verify(kv, bt, torch.tensor([57 + at], dtype=torch.int32, device=DEV),
                                            torch.as_tensor(cand, device=DEV),
                                            n_valid=torch.tensor([n], dtype=torch.int32, device=DEV),
                                            dump_seq_ids=dump)
            torch.cuda.synchronize()
            assert int(status[0]) == 0
            rows.append(logits[0, :n].cpu())
            at += n
        k, v = gpu_kv_tokens(kv, bt[0], 57 + 24, shape.head_dim)
        return torch.cat(rows), k, v

    ref = run([24], 24)
    for cuts, window in (([8, 8, 8], 8), ([1] * 24, 1), ([5, 19], 32), ([17, 7], 64), ([3, 16, 5], 16)):
        got = run(cuts, window)
        for a, b in zip(ref, got):
            assert torch.equal(a, b), cuts
    assert torch.isfinite(ref[0]).all()


def test_split_into_wide_windows_does_not_matter_either(env):
    """The same for windows beyond 64 rows (up to the largest, 512)."""
    shape, w, sess = env
    rng = wl.rng_for(42, 15)
    prompt = wl.random_tokens(rng, 41, shape.vocab)
    tokens = wl.random_tokens(rng, 300, shape.vocab)
    table, num_blocks = wl.make_block_table(rng, [41 + 300], 16, spare_blocks=1)
    bt = torch.as_tensor(table, device=DEV)
    dump = torch.zeros(1, dtype=torch.int32, device=DEV)

    def run(cuts, window):
        kv = sess.kv_cache(num_blocks, fill=float("nan"))
        sess.prefill(kv, bt, [prompt], window=32)
        rows, at = [], 0
        for n in cuts:
            cand = np.zeros((1, window), dtype=np.int32)
            cand[0, :n] = tokens[at:at + n]
            _, status, logits = sess.verify(kv, bt, torch.tensor([41 + at], dtype=torch.int32, device=DEV),
                                            torch.as_tensor(cand, device=DEV),
                                            n_valid=torch.tensor([n], dtype=torch.int32, device=DEV),
                                            dump_seq_ids=dump)
            torch.cuda.synchronize()
            assert int(status[0]) == 0
            rows.append(logits[0, :n].cpu())
            at += n
        k, v = gpu_kv_tokens(kv, bt[0], 41 + 300, shape.head_dim)
        return torch.cat(rows), k, v

    ref = run([64, 64, 64, 64, 44], 64)
    for cuts, window in (([300], 300), ([300], 512), ([128, 172], 256), ([200, 100], 200)):
        got = run(cuts, window)
        for a, b in zip(ref, got):
            assert torch.equal(a, b), cuts
    assert torch.isfinite(ref[0]).all()


def test_many_short_sequences_without_a_merge_pass(env):
    """From 128 (sequence, kv head) pairs whose contexts fit one 2048-key unit the attention kernel writes its
    output itself; rows and sequences that take no part get zeros once per call.  Every live sequence must give
    bitwise what it gives alone (where the partials go through the merge pass), ragged and bad neighbours or not."""
    shape, w, sess = env
    rng = wl.rng_for(42, 16)
    window, n_seq = 8, 70
    lens = wl.uniform_lengths(rng, n_seq, 5, 300)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in lens]
    table, num_blocks = wl.make_block_table(rng, lens + window, 16, spare_blocks=3)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks, fill=float("nan"))
    sess.prefill(kv, bt, prompts, window=16)
    cand = wl.random_tokens(rng, n_seq * window, shape.vocab).reshape(n_seq, window).astype(np.int32)
    n_valid = rng.integers(1, window + 1, size=n_seq).astype(np.int32)
    n_valid[[0, 33, 69]] = window
    cand[11, 2] = shape.vocab                      # a sequence that is switched off
    n_valid[11] = window
    sample = [0, 33, 69, 20]
    d = lambda a: torch.as_tensor(a, device=DEV)
    out, status, logits = sess.verify(kv, bt, d(lens), d(cand), n_valid=d(n_valid),
                                      dump_seq_ids=torch.tensor(sample, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    want = [0] * n_seq
    want[11] = B.LLM42_SEQ_BAD_TOKEN
    assert status.tolist() == want and bool((out[11] == -1).all())
    for j, s in enumerate(sample):
        n = int(n_valid[s])
        assert torch.isfinite(logits[j, :n]).all()
        o1, st1, lg1 = sess.verify(kv, bt[s:s + 1].contiguous(), d(lens[s:s + 1]), d(cand[s:s + 1]), n_valid=d(n_valid[s:s + 1]),
                                   dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert torch.equal(lg1[0, :n], logits[j, :n]) and torch.equal(o1[0], out[s]), s


def test_more_sequence_head_pairs_than_one_grid_axis_holds(env):
    """40 000 sequences of one row each (the width of a decoding step, on the fixed schedule): 80 000 (sequence,
    kv head) pairs, more than a launch can number on its second grid axis, and 40 192 padded rows through every
    GEMM, the attention partials folded by the merge pass.  Sampled sequences must give bitwise what they give alone."""
    shape, w, sess = env
    rng = wl.rng_for(42, 21)
    n_seq = 40000
    lens = rng.integers(0, 41, size=n_seq).astype(np.int32)
    # a table wide enough for 2080 positions: two 2048-key units per sequence, so the partials go through the merge pass
    table, num_blocks = wl.make_block_table(rng, lens + 1, 16, max_blocks_per_seq=130, spare_blocks=2)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(5))
    cand = wl.random_tokens(rng, n_seq, shape.vocab).reshape(n_seq, 1).astype(np.int32)
    sample = [0, 1, 17, 20001, 39999]
    d = lambda a: torch.as_tensor(a, device=DEV)
    out, status, logits = sess.verify(kv, bt, d(lens), d(cand), dump_seq_ids=torch.tensor(sample, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert int(status.max()) == 0 and int(out.min()) >= 0 and torch.isfinite(logits).all()
    for j, s in enumerate(sample):
        o1, st1, lg1 = sess.verify(kv, bt[s:s + 1].contiguous(), d(lens[s:s + 1]), d(cand[s:s + 1]),
                                   dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert torch.equal(lg1[0], logits[j]) and torch.equal(o1[0], out[s]), s


def test_whole_sequences_as_attention_items_or_not(env):
    """With two or more (sequence, kv head) workgroups per CU and contexts beyond one 2048-key super the plan kernel
    may hand whole sequences to the attention workgroups (supers folded in registers, no merge pass) - if the lengths
    of the call deal out evenly, which it decides on the device.  Two calls of 1024 sequences x 64 rows (four items
    per workgroup): lengths that balance, and one long sequence among short ones (which falls back to per-super
    items).  Either way sampled
    sequences give bitwise what they give alone, where the partials go through the merge pass."""
    shape, w, sess = env
    window, n_seq = 64, 1024
    d = lambda a: torch.as_tensor(a, device=DEV)
    for case, seed in (("even", 31), ("one long", 32)):
        rng = wl.rng_for(42, seed)
        lens = rng.integers(2000, 2200, size=n_seq).astype(np.int32) if case == "even" else \
            rng.integers(3, 200, size=n_seq).astype(np.int32)
        if case == "one long":
            lens[5] = 2150
        table, num_blocks = wl.make_block_table(rng, lens + window, 16, max_blocks_per_seq=2304 // 16, spare_blocks=2)
        bt = d(table)
        kv = sess.kv_cache(num_blocks)
        kv.normal_(generator=torch.Generator(device=DEV).manual_seed(seed))
        cand = wl.random_tokens(rng, n_seq * window, shape.vocab).reshape(n_seq, window).astype(np.int32)
        n_valid = rng.integers(1, window + 1, size=n_seq).astype(np.int32)
        n_valid[[0, 5, 1023]] = window
        sample = [0, 5, 600, 1023]
        out, status, logits = sess.verify(kv, bt, d(lens), d(cand), n_valid=d(n_valid),
                                          dump_seq_ids=torch.tensor(sample, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert int(status.max()) == 0, case
        for j, s_ in enumerate(sample):
            n = int(n_valid[s_])
            assert torch.isfinite(logits[j, :n]).all(), (case, s_)
            o1, st1, lg1 = sess.verify(kv, bt[s_:s_ + 1].contiguous(), d(lens[s_:s_ + 1]), d(cand[s_:s_ + 1]),
                                       n_valid=d(n_valid[s_:s_ + 1]), dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV))
            torch.cuda.synchronize()
            assert torch.equal(lg1[0, :n], logits[j, :n]) and torch.equal(o1[0], out[s_]), (case, s_)
        del kv


def test_stale_and_poisoned_slots_are_never_read(env):
    """Slots at or beyond the committed length hold fast-path leftovers; whatever bit
    patterns they contain (including NaN) the result is the same, and the window's
    slots hold the verifier's values afterwards."""
    shape, w, sess = env
    rng = wl.rng_for(42, 6)
    prompt = wl.random_tokens(rng, 45, shape.vocab)        # 45: the window starts inside a block
    win = wl.random_tokens(rng, 8, shape.vocab)
    clean = _batch(sess, shape, [prompt], [win], 8, 0, seed=7, kv_fill=0.0)
    for poison in (float("nan"), float("inf"), -3.0e38):
        dirty = _batch(sess, shape, [prompt], [win], 8, 0, seed=7, kv_fill=poison)
        for a, b in zip(clean, dirty):
            assert torch.equal(a, b), poison
    # shorter n_valid: rows beyond it are padding and their slots stay untouched
    part = _batch(sess, shape, [prompt], [win], 8, 0, seed=7, kv_fill=float("nan"), n_valid=[5])
    assert torch.equal(part[0][:5], clean[0][:5])
    assert torch.equal(part[1][:, :5], clean[1][:, :5]) and torch.isnan(part[1][:, 5:]).all()
    assert part[3][:5].tolist() == clean[3][:5].tolist() and part[3][5:].tolist() == [-1, -1, -1]


def test_long_context_over_several_attention_chunks(env):
    """Context of 1035 keys: five 256-key chunk partials are merged; checked against the
    checker and for invariance to batch company.  (Contexts past a 2048-key super: test_gpu_attention_modes.py.)"""
    shape, w, sess = env
    cfg = oracle_cfg(shape)
    rng = wl.rng_for(42, 8)
    prompt = wl.random_tokens(rng, 1019, shape.vocab)      # window 1019..1034 straddles position 1024
    win = wl.random_tokens(rng, 16, shape.vocab)
    okv = orc.OracleKV(cfg, 1019 + 16)
    orc.forward_window(cfg, w, okv, 0, prompt)
    o_logits = orc.forward_window(cfg, w, okv, 1019, win)
    alone = _batch(sess, shape, [prompt], [win], 16, 0, seed=9)
    assert_logits_close(alone[0], o_logits, "long context")
    assert float((alone[1] - okv.k[:, 1019:]).abs().max()) < 2e-2
    other = wl.random_tokens(rng, 2100, shape.vocab)
    company = _batch(sess, shape, [other, prompt], [win[::-1].copy(), win], 16, 1, seed=10)
    for a, b in zip(alone, company):
        assert torch.equal(a, b)


def test_bad_sequences_are_skipped_and_do_not_disturb_the_others(env):
    shape, w, sess = env
    rng = wl.rng_for(42, 11)
    window = 8
    prompts = [wl.random_tokens(rng, n, shape.vocab) for n in (30, 41, 52, 23)]
    wins = [wl.random_tokens(rng, window, shape.vocab) for _ in range(4)]
    good = _batch(sess, shape, [prompts[1]], [wins[1]], window, 0, seed=12)
    lens = np.array([30, 41, 52, 23], dtype=np.int32)
    table, num_blocks = wl.make_block_table(rng, lens + window, 16, spare_blocks=2)
    bt_host = table.copy()
    kv = sess.kv_cache(num_blocks, fill=0.0)
    sess.prefill(kv, torch.as_tensor(table, device=DEV), prompts, window=16)
    before = kv.clone()
    cand = np.stack(wins).astype(np.int32)
    cand[0, 3] = shape.vocab                 # token id out of range
    bt_host[2, 1] = num_blocks + 5           # block id out of range
    seq_lens = lens.copy()
    seq_lens[3] = -4                         # negative length
    d = lambda a: torch.as_tensor(a, device=DEV)
    sl = d(seq_lens)
    out, status, logits = sess.verify(kv, d(bt_host), sl, d(cand),
                                      dump_seq_ids=torch.tensor([1], dtype=torch.int32, device=DEV))
    counts, toks, rolled = sess.commit(d(cand), out, sl)
    torch.cuda.synchronize()
    assert status.tolist() == [B.LLM42_SEQ_BAD_TOKEN, 0, B.LLM42_SEQ_BAD_BLOCK, B.LLM42_SEQ_BAD_LENGTH]
    assert torch.equal(logits[0].cpu(), good[0])
    assert bool((out[[0, 2, 3]] == -1).all()) and bool((out[1] >= 0).all())
    assert counts.tolist()[0] == 0 and counts.tolist()[2] == 0 and counts.tolist()[3] == 0 and counts.tolist()[1] >= 1
    assert sl.tolist()[0] == 30 and sl.tolist()[2] == 52 and sl.tolist()[3] == -4
    # the skipped sequences' cache blocks were not written
    for s in (0, 2, 3):
        ids = torch.as_tensor(table[s][table[s] >= 0], device=DEV).long()
        assert torch.equal(kv[:, :, ids].view(torch.int16), before[:, :, ids].view(torch.int16))


def test_host_side_errors(env):
    shape, w, sess = env
    d = lambda a, t=torch.int32: torch.as_tensor(a, dtype=t, device=DEV)
    kv = sess.kv_cache(4)
    bt = d([[0, 1]])
    ok = dict(kv=kv, block_table=bt, seq_lens=d([3]), candidates=d([[1, 2, 3, 4]]))
    with pytest.raises(B.Llm42Error) as e:
        sess.verify(max_context=64, **ok)                      # 64 > 2 blocks * 16
    assert e.value.status == B.LLM42_ECAPACITY
    with pytest.raises(B.Llm42Error) as e:
        sess.verify(max_context=4000, kv=kv, block_table=d(np.zeros((1, 300))), seq_lens=d([3]),
                    candidates=d([[1, 2, 3, 4]]))              # beyond max_position
    assert e.value.status == B.LLM42_ECAPACITY
    with pytest.raises(B.Llm42Error) as e:
        B.llm42_verify_window(sess.model, kv, 4, bt, d([3]), d([[1, 2, 3, 4]]), 4, None, 32,
                              torch.empty((1, 4), dtype=torch.int32, device=DEV),
                              torch.empty(512, dtype=torch.uint8, device=DEV))
    assert e.value.status == B.LLM42_EWORKSPACE
    with pytest.raises(B.Llm42Error) as e:
        B.llm42_workspace_bytes(sess.model, 1, B.LLM42_MAX_WINDOW + 1, 128)
    assert e.value.status == B.LLM42_EINVAL
    with pytest.raises(B.Llm42Error) as e:
        B.llm42_workspace_bytes(sess.model, B.LLM42_MAX_ROWS // 2 + 1, 2, 128)      # more rows than one call takes
    assert e.value.status == B.LLM42_EINVAL
    with pytest.raises(ValueError):                                                  # a KV tensor too small for num_blocks
        B.llm42_verify_window(sess.model, kv, 5, bt, d([3]), d([[1, 2, 3, 4]]), 4, None, 32,
                              torch.empty((1, 4), dtype=torch.int32, device=DEV), sess.workspace(1, 4, 32))
