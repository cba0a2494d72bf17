"""Seeded stochastic sampling on the GPU (paper section 4.4 "Sampling") against the checker's
sampler, and the properties that make it usable under the verify-rollback protocol: the sample is
a function of (seed, request, position, logits) only, so it is the same in any batch, slot or
window split, and the decode - verify - rollback loop reproduces the verifier-only stream."""
import numpy as np
import pytest
import torch

from helpers import orc, wl
from gpu_helpers import Scenario, VerifierSession, oracle_kv_to_gpu
from paper_2601_17768_amd import binding as B, dvr

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
    rng = wl.rng_for(42, 21)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in (16, 40, 64, 29)]
    return Scenario(shape, w, prompts, window=8, rate=0.10, seed=42)


def _gpu_state(sess, sc, order=None):
    order = list(range(len(sc.lens))) if order is None else order
    lens = sc.lens[order]
    table, num_blocks = wl.make_block_table(wl.rng_for(42, 22 + len(order)), lens + sc.window, 16, spare_blocks=3)
    kv = sess.kv_cache(num_blocks)
    bt = torch.as_tensor(table, device=DEV)
    for slot, s in enumerate(order):
        oracle_kv_to_gpu(kv, bt[slot], sc.okv[s], int(sc.lens[s]))
    return kv, bt, torch.as_tensor(lens, device=DEV), torch.as_tensor(sc.candidates[order], device=DEV)


def test_sampled_tokens_match_the_checker_where_decidable(tiny, scenario):
    shape, w, sess = tiny
    sc = scenario
    temperature, seed = 0.8, 20260117
    rids = torch.tensor([1001, 7, 1 << 40, 12345678901], dtype=torch.int64, device=DEV)
    kv, bt, lens, cand = _gpu_state(sess, sc)
    dump = torch.arange(4, dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, lens, cand, dump_seq_ids=dump,
                                      sampling=B.make_sampling(temperature, seed, rids))
    torch.cuda.synchronize()
    assert status.tolist() == [0] * 4
    _, o_logits = sc.oracle_verify()
    decided = 0
    for s in range(4):
        pos = [int(sc.lens[s]) + i for i in range(sc.window)]
        toks, noisy = orc.sample_tokens(o_logits[s], temperature, seed, int(rids[s]), pos)
        err = (logits[s].cpu().double() - o_logits[s]).abs().max(dim=-1).values / temperature + 1e-4
        margin = orc.top2_margin(noisy)
        for i in range(sc.window):
            if float(margin[i]) > 2 * float(err[i]):          # no reordering of the perturbed top is possible
                assert int(out[s, i]) == int(toks[i]), f"seq {s} row {i}"
                decided += 1
    assert decided >= 28                                      # nearly every row is decidable at these margins
    # and the sampler really is stochastic: it leaves the arg-max on a good part of the rows
    greedy, _, _ = sess.verify(*_gpu_state(sess, sc))
    assert int((greedy != out).sum()) >= 8


def test_sample_is_independent_of_batch_slot_and_window_split(tiny, scenario):
    shape, w, sess = tiny
    sc = scenario
    sp = lambda ids: B.make_sampling(1.0, 99, torch.tensor(ids, dtype=torch.int64, device=DEV))
    kv, bt, lens, cand = _gpu_state(sess, sc)
    base, _, _ = sess.verify(kv, bt, lens, cand, sampling=sp([50, 51, 52, 53]))
    base = base.clone()
    # other slots, other companions: request ids travel with the sequences
    order = [2, 0]
    kv, bt, lens, cand = _gpu_state(sess, sc, order)
    out, _, _ = sess.verify(kv, bt, lens, cand, sampling=sp([52, 50]))
    assert torch.equal(out[0], base[2]) and torch.equal(out[1], base[0])
    # the same positions verified as two windows of 4: same samples (keyed by absolute position)
    kv, bt, lens, cand = _gpu_state(sess, sc)
    c4 = cand[:, :4].contiguous()
    first, _, _ = sess.verify(kv, bt, lens, c4, sampling=sp([50, 51, 52, 53]))
    assert torch.equal(first, base[:, :4])
    second, _, _ = sess.verify(kv, bt, lens + 4, cand[:, 4:].contiguous(), sampling=sp([50, 51, 52, 53]))
    assert torch.equal(second, base[:, 4:])
    # another seed, another request id: other samples; temperature 0: the arg-max
    kv, bt, lens, cand = _gpu_state(sess, sc)
    other, _, _ = sess.verify(kv, bt, lens, cand, sampling=B.make_sampling(1.0, 100, None))
    assert int((other != base).sum()) >= 8
    greedy, _, _ = sess.verify(kv, bt, lens, cand)
    zero, _, _ = sess.verify(kv, bt, lens, cand, sampling=B.make_sampling(0.0, 99, None))
    assert torch.equal(zero, greedy)


def test_loop_with_sampling_reproduces_the_verifier_only_stream(tiny):
    shape, w, sess = tiny
    rng = wl.rng_for(42, 30)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in rng.integers(16, 64, size=20)]
    new, window = 40, 8

    def state(group):
        lens = np.array([len(p) for p in group], dtype=np.int32)
        table, nb = wl.make_block_table(wl.rng_for(42, 31), lens + new + 3 * window, 16, spare_blocks=2)
        kv = sess.kv_cache(nb)
        bt = torch.as_tensor(table, device=DEV)
        first = sess.prefill(kv, bt, group, window=32)
        return kv, bt, torch.as_tensor(lens, device=DEV), first

    ids = torch.arange(900, 920, dtype=torch.int64, device=DEV)
    kv, bt, lens, first = state(prompts[:1])
    ref = dvr.generate_verifier_only(sess, kv, bt, lens, first, new, sampling=B.make_sampling(0.9, 5, ids[:1]))[0]
    kv, bt, lens, first = state(prompts)
    toks, st = dvr.generate(sess, kv, bt, lens, first, new, window, sampling=B.make_sampling(0.9, 5, ids))
    print(f"{st.iterations} iterations, {st.rolled_back} candidates rolled back", flush=True)
    assert torch.equal(toks[0], ref)
    greedy_ref = dvr.generate_verifier_only(sess, *state(prompts[:1]), new)[0]
    assert not torch.equal(ref, greedy_ref)
