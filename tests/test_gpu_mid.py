"""GPU parity at the 8B model's layer widths (d 4096, 32 q / 8 kv heads of 128, FFN
14336) with 2 layers and a 32064-entry vocabulary, sized so that the checker
finishes in seconds while every kernel runs at its real tile shapes: several
feature tiles, window 32, ragged contexts, scattered KV blocks."""
import numpy as np
import pytest
import torch

from helpers import orc, wl
from gpu_helpers import Scenario, VerifierSession, assert_logits_within_noise, checker_noise, REL_TOL, oracle_kv_to_gpu, gpu_kv_tokens, assert_tokens_match_where_decidable, ABS_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def as_dtype(w, dtype):
    out = {k: w[k].to(dtype) for k in ("embed", "final_norm", "lm_head")}
    out["layers"] = [{k: v.to(dtype) for k, v in lw.items()} for lw in w["layers"]]
    return out


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n_layers", [1, 2])
def test_mid_shape_against_checker(n_layers):
    """One layer: nothing amplifies a rounding difference yet, and still the checker's own noise (printed) reaches
    the benchmark spec's 2e-2; the relative bound (1e-2 of the largest logit) holds and is asserted literally."""
    shape = wl.LLAMA_8B.replace(n_layers=n_layers, vocab=32064)
    w = wl.make_weights(shape, seed=43)
    sess = VerifierSession(shape, w, max_position=1024, device=DEV)
    rng = wl.rng_for(43, 1)
    prompts = [wl.random_tokens(rng, n, shape.vocab) for n in (70, 150, 301)]
    window = 32
    sc = Scenario(shape, as_dtype(w, torch.float64), prompts, window=window, rate=0.05, seed=43)
    table, num_blocks = wl.make_block_table(rng, sc.lens + window, 16, spare_blocks=5)
    bt = torch.as_tensor(table, device=DEV)
    kv = sess.kv_cache(num_blocks, fill=float("nan"))
    for s, okv in enumerate(sc.okv):
        oracle_kv_to_gpu(kv, bt[s], okv, int(sc.lens[s]))
    seq_lens = torch.as_tensor(sc.lens, device=DEV)
    cand = torch.as_tensor(sc.candidates, device=DEV)
    dump = torch.arange(3, dtype=torch.int32, device=DEV)
    out, status, logits = sess.verify(kv, bt, seq_lens, cand, dump_seq_ids=dump)
    counts, toks, rolled = sess.commit(cand, out, seq_lens)
    torch.cuda.synchronize()
    assert status.tolist() == [0, 0, 0]
    o_tokens, o_logits = sc.oracle_verify()
    # the checker's own noise on these inputs: float32 accumulation and rounded softmax weights against the definition
    w32 = as_dtype(w, torch.float32)
    noise = torch.cat([checker_noise(sc.cfg, w32, sc.okv[s].k, sc.okv[s].v, int(sc.lens[s]), sc.candidates[s], o_logits[s])
                       for s in range(3)])
    noise_rms, noise_max = float((noise * noise).mean().sqrt()), float(noise.max())
    print(f"{n_layers} layer(s): checker noise rms {noise_rms:.3e} max {noise_max:.3e}")
    exempt = 0
    for s in range(3):
        err, rms = assert_logits_within_noise(logits[s], o_logits[s], noise_rms, noise_max, f"{n_layers}-layer shape seq {s}")
        assert err <= REL_TOL * float(o_logits[s].abs().max())           # spec relative bound, literally
        margin = orc.top2_margin(o_logits[s])
        seq_exempt = assert_tokens_match_where_decidable(out[s].cpu(), logits[s], o_tokens[s], o_logits[s], f"seq {s}")
        exempt += seq_exempt
        L = int(sc.lens[s])
        gk, gv = gpu_kv_tokens(kv, bt[s], L + window, shape.head_dim)
        assert float((gk[:, L:] - sc.okv[s].k[:, L:L + window]).abs().max()) < 0.05
        assert float((gv[:, L:] - sc.okv[s].v[:, L:L + window]).abs().max()) < 0.05
        c, t, r = orc.commit_rollback(sc.candidates[s], out[s].tolist(), window)
        assert (int(counts[s]), int(rolled[s])) == (c, r) and int(seq_lens[s]) == L + c
        if seq_exempt == 0:
            assert (c, t, r) == orc.commit_rollback(sc.candidates[s], o_tokens[s], window)
    print(f"rows exempt from the exact-token check (margin <= 2 x row error): {exempt} of {3 * window}")
    # the same three sequences one by one: bitwise the same logits (batch invariance at real widths)
    for s in range(3):
        kv1 = sess.kv_cache(num_blocks, fill=0.0)
        oracle_kv_to_gpu(kv1, bt[s], sc.okv[s], int(sc.lens[s]))   # note: window slots of okv were rewritten; prefix only
        _, st1, lg1 = sess.verify(kv1, bt[s:s + 1].contiguous(), torch.as_tensor(sc.lens[s:s + 1], device=DEV),
                                  cand[s:s + 1].contiguous(), dump_seq_ids=torch.zeros(1, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert torch.equal(lg1[0], logits[s])
    sess.close()
