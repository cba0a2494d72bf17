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
