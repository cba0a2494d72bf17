"""llm42_prefill (deterministic prefill, paper section 4.1 on observation O3 and section 4.2 on the first
output token): the call equals the same windows pushed through llm42_verify_window from the host,
bit for bit, whatever the chunk; a cached prefix can be shared between sequences (which the
limitations paragraph at the end of section 5 says the prototype cannot do); and its error reporting.
Parity of the prefilled cache and first token with the checker is in test_gpu_tiny."""
import numpy as np
import pytest
import torch

from helpers import wl
from gpu_helpers import VerifierSession
from paper_2601_17768_amd import binding as B
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


def _kv_bits(kv, bt_row, length, head_dim):
    k, v = kv_layout.read_tokens(kv, bt_row, length, head_dim)
    return k.view(torch.int16).cpu(), v.view(torch.int16).cpu()


def test_prefill_equals_the_windows_driven_from_the_host_for_any_chunk(tiny):
    shape, w, sess = tiny
    rng = wl.rng_for(201, 1)
    lens = np.array([1, 7, 16, 33, 64, 100, 129], dtype=np.int32)
    prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in lens]
    table, num_blocks = wl.make_block_table(wl.rng_for(201, 2), lens + 8, 16, spare_blocks=4)
    bt = torch.as_tensor(table, device=DEV)

    kv_ref = sess.kv_cache(num_blocks, fill=float("nan"))
    first_ref = sess.prefill_by_windows(kv_ref, bt, prompts, window=8)
    torch.cuda.synchronize()
    ref = [_kv_bits(kv_ref, bt[s], int(lens[s]), shape.head_dim) for s in range(len(lens))]
    for chunk in (8, 1, 32, 64):
        if chunk == 1:
            sel = [0, 1, 2]                     # one row per pass: keep it short
        else:
            sel = list(range(len(lens)))
        kv = sess.kv_cache(num_blocks, fill=float("nan"))
        first = sess.prefill(kv, bt[sel].contiguous(), [prompts[s] for s in sel], window=chunk)
        torch.cuda.synchronize()
        assert first.tolist() == first_ref[sel].tolist(), f"chunk {chunk}"
        for j, s in enumerate(sel):
            k, v = _kv_bits(kv, bt[s], int(lens[s]), shape.head_dim)
            assert torch.equal(k, ref[s][0]) and torch.equal(v, ref[s][1]), f"chunk {chunk}, sequence {s}"


def test_a_cached_prefix_is_shared_between_sequences(tiny):
    shape, w, sess = tiny
    rng = wl.rng_for(202, 1)
    common = wl.random_tokens(rng, 48, shape.vocab)                      # three whole blocks
    tail_a, tail_b = wl.random_tokens(rng, 22, shape.vocab), wl.random_tokens(rng, 37, shape.vocab)
    a, b = np.concatenate([common, tail_a]), np.concatenate([common, tail_b])
    num_blocks = 32
    # sequence A owns blocks 3, 9, 4 for the prefix; B's table starts with the same three blocks
    bt_a = torch.tensor([[3, 9, 4, 11, 12, 13, 14, 15]], dtype=torch.int32, device=DEV)
    bt_b = torch.tensor([[3, 9, 4, 20, 21, 22, 23, 24]], dtype=torch.int32, device=DEV)
    bt_alone = torch.tensor([[1, 2, 5, 6, 7, 8, 10, 16]], dtype=torch.int32, device=DEV)
    kv = sess.kv_cache(num_blocks, fill=float("nan"))
    first_a = sess.prefill(kv, bt_a, [a], window=16)
    # B: only what follows the shared prefix is computed
    first_b = sess.prefill(kv, bt_b, [tail_b], window=16, cached=torch.tensor([48], dtype=torch.int32, device=DEV))
    # reference: B from scratch in blocks of its own
    kv2 = sess.kv_cache(num_blocks, fill=float("nan"))
    first_b_alone = sess.prefill(kv2, bt_alone, [b], window=16)
    first_a_alone = sess.prefill(kv2, bt_a, [a], window=32)
    torch.cuda.synchronize()
    assert first_b.tolist() == first_b_alone.tolist() and first_a.tolist() == first_a_alone.tolist()
    k, v = _kv_bits(kv, bt_b[0], len(b), shape.head_dim)
    k2, v2 = _kv_bits(kv2, bt_alone[0], len(b), shape.head_dim)
    assert torch.equal(k, k2) and torch.equal(v, v2)


def test_flagged_and_empty_prompts(tiny):
    shape, w, sess = tiny
    rng = wl.rng_for(203, 1)
    good = wl.random_tokens(rng, 20, shape.vocab)
    bad_token = good.copy()
    bad_token[13] = shape.vocab                                          # outside the vocabulary, in the second pass
    too_long = wl.random_tokens(rng, 40, shape.vocab)                     # longer than max_prompt_len below
    prompts = [good, bad_token, np.zeros(0, dtype=np.int32), too_long, good]
    lens = np.array([len(p) for p in prompts], dtype=np.int32)
    offsets = np.zeros(len(prompts) + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(lens)
    table, num_blocks = wl.make_block_table(wl.rng_for(203, 2), np.maximum(lens, 1) + 8, 16, spare_blocks=2)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks, fill=float("nan"))
    n = len(prompts)
    chunk, max_context = 8, 48
    ws = torch.empty(B.llm42_prefill_workspace_bytes(sess.model, n, chunk, max_context), dtype=torch.uint8, device=DEV)
    first = torch.full((n,), 12345, dtype=torch.int32, device=DEV)
    status = torch.full((n,), 99, dtype=torch.int32, device=DEV)
    d = lambda x: torch.as_tensor(x, device=DEV)
    B.llm42_prefill(sess.model, kv, num_blocks, bt, torch.zeros(n, dtype=torch.int32, device=DEV),
                    d(np.concatenate(prompts).astype(np.int32)), d(offsets), 24, chunk, max_context, first, ws, status)
    torch.cuda.synchronize()
    assert status.tolist() == [0, B.LLM42_SEQ_BAD_TOKEN, 0, B.LLM42_SEQ_BAD_LENGTH, 0]
    f = first.tolist()
    assert f[1] == -1 and f[2] == -1 and f[3] == -1
    assert f[0] == f[4] and 0 <= f[0] < shape.vocab                      # the healthy sequences are not disturbed
    kv_ref = sess.kv_cache(num_blocks, fill=float("nan"))
    ref = sess.prefill(kv_ref, bt[:1].contiguous(), [good], window=chunk)
    assert ref.tolist() == [f[0]]
    # host-side argument checks
    with pytest.raises(B.Llm42Error):
        B.llm42_prefill(sess.model, kv, num_blocks, bt, torch.zeros(n, dtype=torch.int32, device=DEV),
                        d(np.concatenate(prompts).astype(np.int32)), d(offsets), 24, 0, max_context, first, ws, status)
    with pytest.raises(B.Llm42Error):
        B.llm42_prefill(sess.model, kv, num_blocks, bt, torch.zeros(n, dtype=torch.int32, device=DEV),
                        d(np.concatenate(prompts).astype(np.int32)), d(offsets), 24, chunk, max_context, first,
                        ws[:1024], status)
