"""llm42_verify_window_static: the verifier pass in the library's built-in scratch area, for callers that
cannot allocate.  Called through the C ABI and compared bit for bit with llm42_verify_window (same kernels, same
schedule) on two calls in a row, the second with a smaller input, so that what the first call left in the area
is there when the second runs."""
import numpy as np
import pytest
import torch

from helpers import wl
from gpu_helpers import VerifierSession, gpu_kv_tokens
from paper_2601_17768_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(sess, shape, rng, n_seq, window, lo, hi):
    lens = wl.uniform_lengths(rng, n_seq, lo, hi)
    table, num_blocks = wl.make_block_table(rng, lens + window, 16, spare_blocks=2)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks)
    kv.normal_(generator=torch.Generator(device=DEV).manual_seed(int(lens.sum())))
    cand = torch.as_tensor(wl.random_tokens(rng, n_seq * window, shape.vocab).reshape(n_seq, window).astype(np.int32),
                           device=DEV)
    n_valid = torch.as_tensor(rng.integers(1, window + 1, size=n_seq).astype(np.int32), device=DEV)
    return kv, num_blocks, bt, torch.as_tensor(lens, device=DEV), cand, n_valid, int(lens.max()) + window


def _both_ways(sess, shape, case, window):
    kv, num_blocks, bt, lens, cand, n_valid, max_context = case
    n_seq = lens.numel()
    dump = torch.arange(n_seq, dtype=torch.int32, device=DEV)
    results = []
    for static in (False, True):
        kv_run = kv.clone()
        out = torch.full((n_seq, window), -7, dtype=torch.int32, device=DEV)
        status = torch.full((n_seq,), -7, dtype=torch.int32, device=DEV)
        logits = torch.zeros((n_seq, window, shape.vocab), dtype=torch.float32, device=DEV)
        if static:
            B.llm42_verify_window_static(sess.model, kv_run, num_blocks, bt, lens, cand, window, n_valid, max_context,
                                         out, status, logits, dump)
        else:
            B.llm42_verify_window(sess.model, kv_run, num_blocks, bt, lens, cand, window, n_valid, max_context, out,
                                  sess.workspace(n_seq, window, max_context), status, logits, dump)
        torch.cuda.synchronize()
        results.append((out, status, logits, kv_run))
    (o0, s0, l0, k0), (o1, s1, l1, k1) = results
    assert s0.tolist() == [0] * n_seq and torch.equal(s0, s1)
    assert torch.equal(o0, o1) and int(o0.max()) >= 0
    assert torch.equal(l0, l1) and torch.isfinite(l0).all()
    assert torch.equal(k0.view(torch.int16), k1.view(torch.int16))


@pytest.mark.timeout(300)
def test_static_scratch_entry_matches_the_workspace_entry_twice_in_a_row():
    shape = wl.TINY
    w = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, w, max_position=4096, device=DEV)
    rng = wl.rng_for(42, 77)
    # first call: 24 sequences x window 16 with contexts past one 2048-key unit (attention partials + merge pass);
    # second call: 3 short sequences x window 8 - a different work split in the same area, smaller everywhere
    _both_ways(sess, shape, _case(sess, shape, rng, 24, 16, 1500, 2500), 16)
    _both_ways(sess, shape, _case(sess, shape, rng, 3, 8, 5, 90), 8)
    # beyond what the area holds (65 280 rows: the fp32 residual stream alone fills it): a clear error, nothing launched
    kv, num_blocks, bt, lens, cand, n_valid, max_context = _case(sess, shape, rng, 2040, 32, 1, 10)
    assert B.llm42_workspace_bytes(sess.model, 2040, 32, max_context) > B.LLM42_STATIC_SCRATCH_BYTES
    out = torch.full((2040, 32), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(B.Llm42Error) as e:
        B.llm42_verify_window_static(sess.model, kv, num_blocks, bt, lens, cand, 32, n_valid, max_context, out)
    assert e.value.status == B.LLM42_EWORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == -7).all())
    sess.close()
