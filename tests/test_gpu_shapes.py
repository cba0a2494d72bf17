"""GPU parity against the checker at head groupings the other tests do not use: one query head per kv
head (head_dim 64) and eight per kv head with head_dim 128 and an attention width (n_q_heads x head_dim)
that differs from d_model; windows below and above the 8 row blocks per (sequence, kv head) at which the
attention switches kernels."""
import numpy as np
import pytest
import torch

from helpers import orc, wl
from gpu_helpers import (Scenario, VerifierSession, assert_logits_close, oracle_kv_to_gpu, gpu_kv_tokens,
                         assert_tokens_match_where_decidable)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = {
    "one query head per kv head": wl.ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                                                 d_ffn=688, vocab=1024, rope_theta=1e4),
    "eight query heads per kv head": wl.ModelShape(n_layers=2, d_model=256, n_q_heads=8, n_kv_heads=1, head_dim=128,
                                                    d_ffn=320, vocab=2048, rope_theta=5e5),
}


@pytest.mark.parametrize("name", sorted(SHAPES))
@pytest.mark.parametrize("window", [8, 24])
def test_head_groupings_against_checker(name, window):
    shape = SHAPES[name]
    w = wl.make_weights(shape, seed=44)
    sess = VerifierSession(shape, w, max_position=512, device=DEV)
    try:
        rng = wl.rng_for(44, window)
        lens = wl.uniform_lengths(rng, 3, 5, 300)
        prompts = [wl.random_tokens(rng, int(n), shape.vocab) for n in lens]
        sc = Scenario(shape, w, prompts, window=window, rate=0.10, seed=44)
        table, num_blocks = wl.make_block_table(rng, sc.lens + window, 16, spare_blocks=3)
        bt = torch.as_tensor(table, device=DEV)
        kv = sess.kv_cache(num_blocks, fill=float("nan"))
        for s, okv in enumerate(sc.okv):
            oracle_kv_to_gpu(kv, bt[s], okv, int(sc.lens[s]))
        seq_lens = torch.as_tensor(sc.lens, device=DEV)
        cand = torch.as_tensor(sc.candidates, device=DEV)
        out, status, logits = sess.verify(kv, bt, seq_lens, cand, dump_seq_ids=torch.arange(3, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert status.tolist() == [0, 0, 0]
        o_tokens, o_logits = sc.oracle_verify()
        for s in range(3):
            assert_logits_close(logits[s], o_logits[s], f"{name}, window {window}, seq {s}")
            assert_tokens_match_where_decidable(out[s].cpu().numpy(), logits[s], o_tokens[s], o_logits[s], f"seq {s}")
            L = int(sc.lens[s])
            gk, gv = gpu_kv_tokens(kv, bt[s], L + window, shape.head_dim)
            assert float((gk[:, L:] - sc.okv[s].k[:, L:L + window]).abs().max()) < 2e-2
            assert float((gv[:, L:] - sc.okv[s].v[:, L:L + window]).abs().max()) < 2e-2
    finally:
        sess.close()
