"""The decode - verify - rollback loop end to end (paper sections 4.1-4.2, figure of the DVR protocol):
whatever the fast path produces, and however its low bits move with the batch, the committed stream
of a sequence is the one the verifier alone would produce, token for token, in any group."""
import numpy as np
import pytest
import torch

from helpers import wl
from gpu_helpers import VerifierSession
from paper_2601_17768_amd import dvr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
WINDOW, NEW = 8, 48


def _state(sess, shape, prompts, room):
    lens = np.array([len(p) for p in prompts], dtype=np.int32)
    table, num_blocks = wl.make_block_table(wl.rng_for(77, len(prompts)), lens + room, 16, spare_blocks=3)
    kv = sess.kv_cache(num_blocks)
    bt = torch.as_tensor(table, device=DEV)
    first = sess.prefill(kv, bt, prompts, window=32)
    return kv, bt, torch.as_tensor(lens, device=DEV), first


@pytest.mark.timeout(600)
def test_committed_stream_does_not_depend_on_the_group():
    # 8B layer widths, 2 layers: wide enough for the fast path's batch-dependent rounding to flip tokens now and then
    shape = wl.LLAMA_8B.replace(n_layers=2, vocab=32064)
    w = wl.make_weights(shape, seed=44)
    sess = VerifierSession(shape, w, max_position=1024, device=DEV)
    rng = wl.rng_for(44, 3)
    target = wl.random_tokens(rng, 45, shape.vocab)
    others = [wl.random_tokens(rng, int(n), shape.vocab) for n in rng.integers(20, 200, size=23)]
    room = NEW + 3 * WINDOW

    # the reference: the target alone, every token through the verifier
    kv, bt, lens, first = _state(sess, shape, [target], room)
    ref = dvr.generate_verifier_only(sess, kv, bt, lens, first, NEW)[0]

    results = {}
    for name, group in (("alone", [target]), ("first of 24", [target] + others), ("last of 9", others[:8] + [target])):
        kv, bt, lens, first = _state(sess, shape, group, room)
        lens0 = lens.clone()
        toks, st = dvr.generate(sess, kv, bt, lens, first, NEW, WINDOW)
        torch.cuda.synchronize()
        slot = 0 if name != "last of 9" else 8
        results[name] = toks[slot]
        print(f"{name}: {st.iterations} iterations, {st.committed} committed, {st.rolled_back} candidates rolled back "
              f"in {st.rollbacks} windows, {st.fast_tokens} fast-path tokens", flush=True)
        # forward progress and bookkeeping (section 4.2): every window commits at least one token per sequence,
        # and the cached length advanced by exactly the committed count
        assert all(c >= len(group) for c in st.per_iteration_committed)
        assert int((lens - lens0).sum()) == st.committed
        assert st.committed + st.rolled_back == st.verified_rows
    for name, toks in results.items():
        assert torch.equal(toks, ref), f"group '{name}' changed the committed stream"
    sess.close()


def test_loop_on_the_small_configuration_matches_the_verifier_alone():
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, w, max_position=512, device=DEV)
    rng = wl.rng_for(42, 9)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in (16, 33, 64, 20, 47)]
    room = NEW + 3 * WINDOW
    kv, bt, lens, first = _state(sess, shape, prompts, room)
    ref = dvr.generate_verifier_only(sess, kv, bt, lens, first, NEW)
    kv, bt, lens, first = _state(sess, shape, prompts, room)
    toks, st = dvr.generate(sess, kv, bt, lens, first, NEW, WINDOW)
    assert torch.equal(toks, ref)
    assert st.committed + st.rolled_back == st.verified_rows
    sess.close()


def test_committed_stream_is_the_checkers_greedy_stream():
    """The paper's end-to-end claim (section 4.2) against the checker: whatever the group, the stream a sequence
    commits is plain greedy decoding as the CPU checker computes it.  Compared token by token up to the first
    position where the two differ; that position must be one the checker itself cannot decide - its top-1/top-2
    margin there is below twice the logit error of this shape (1e-2: the measured worst case is 7e-3) - and the
    compared prefix must be long enough to mean something."""
    from helpers import orc, oracle_cfg
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    cfg = oracle_cfg(shape)
    sess = VerifierSession(shape, w, max_position=512, device=DEV)
    rng = wl.rng_for(42, 19)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in rng.integers(16, 65, size=20)]
    room = NEW + 3 * WINDOW
    logit_err = 1e-2

    def checker_stream(prompt):
        """Greedy decoding by the checker: tokens and the margin behind each of them."""
        okv = orc.OracleKV(cfg, len(prompt) + NEW + 1)
        lg = orc.forward_window(cfg, w, okv, 0, list(prompt))[-1:]
        toks, margins, L = [], [], len(prompt)
        for _ in range(NEW):
            toks.append(int(orc.greedy_argmax(lg)[0]))
            margins.append(float(orc.top2_margin(lg)[0]))
            lg = orc.forward_window(cfg, w, okv, L, [toks[-1]])
            L += 1
        return toks, margins

    refs = [checker_stream(p) for p in prompts]
    for n_group in (1, 5, 20):
        group = prompts[:n_group]
        kv, bt, lens, first = _state(sess, shape, group, room)
        toks, st = dvr.generate(sess, kv, bt, lens, first, NEW - 1, WINDOW)
        torch.cuda.synchronize()
        agreed = []
        for s in range(n_group):
            ref_toks, margins = refs[s]
            got = [int(first[s])] + toks[s].tolist()          # the first token comes from the prefill
            n = 0
            while n < NEW and got[n] == ref_toks[n]:
                n += 1
            if n < NEW:
                assert margins[n] < 2 * logit_err, (n_group, s, n, margins[n], got[n], ref_toks[n])
            agreed.append(n)
        print(f"group of {n_group}: tokens equal to the checker's greedy stream before the first undecidable "
              f"position: {agreed} of {NEW}; {st.rolled_back} candidates rolled back", flush=True)
        # (measured: 17 of 48 alone; 13 of 20 sequences agree over all 48 tokens, one differs at an undecidable first token)
        assert sum(agreed) >= n_group * NEW // 3
    sess.close()
