"""Writes tests/golden/c2_llama8b_window32.json: the checker's results for the
8B-shape single-sequence configuration (32 layers, d 4096, 32 q / 8 kv heads of 128,
FFN 14336, vocab 128256; one 512-token random prompt, verification window 32,
candidates = greedy continuation with 2 % random replacements, seed 42).

Calls only the CPU checker (oracle/) and the seeded input generator; run it from
the repository root:  python tests/golden/make_c2_golden.py   (about 10 minutes
and 50 GB of host memory).  Stored: the window inputs, the checker's output tokens,
top-2 logits per row, logits at 128 seeded vocabulary columns per row, and a few
K/V cache values of the window, all from the float64 checker.

Also stored ("self_noise"): how far the checker moves when only its accumulation
precision changes (float32 instead of float64, prompt replayed in four windows
instead of one) on the very same inputs, and how far when the softmax weights
are rounded to bf16 as well.  Every bf16 rounding point of the model
turns a last-bit difference in summation order into a one-ulp difference, so two
correct evaluations with bf16 matrix operands decorrelate; these figures are the
measured size of that effect at this depth and are what the GPU test scales its
tolerance by.  `--self-noise-only` recomputes just that part (about 12 minutes).
"""
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import llm42_oracle as orc                      # noqa: E402
from paper_2601_17768_amd import workloads as wl            # noqa: E402

SEED, PROMPT_LEN, WINDOW, RATE, N_COLS = 42, 512, 32, 0.02, 128
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c2_llama8b_window32.json")


def c2_inputs():
    """Seeded inputs of the configuration that do not need the model."""
    shape = wl.LLAMA_8B
    prompt = wl.random_tokens(wl.rng_for(SEED, 2, 0), PROMPT_LEN, shape.vocab)
    cols = np.sort(wl.rng_for(SEED, 2, 1).choice(shape.vocab, size=N_COLS, replace=False)).astype(np.int64)
    return shape, prompt, cols


def self_noise(gold, cfg, w, prompt, cols):
    """The checker against itself on the stored inputs: what moves when a correct evaluation accumulates in
    float32 instead of float64 (prompt replayed in windows of 128 instead of one), and what moves when, in
    addition, the softmax weights are rounded to bf16 before they multiply V (`round_p`, the one rounding point
    a bf16 matrix unit adds to the definition), for two different cuts of the prompt into windows - the spread
    between those two is the error bar of the figure."""
    ref = torch.tensor(gold["logits_at_columns"], dtype=torch.float64)

    def one(round_p, cut):
        kv = orc.OracleKV(cfg, PROMPT_LEN + WINDOW)
        for a in range(0, PROMPT_LEN, cut):
            orc.forward_window(cfg, w, kv, a, prompt[a:a + cut], acc_dtype=torch.float32, round_p=round_p)
        lg = orc.forward_window(cfg, w, kv, PROMPT_LEN, gold["candidates"], acc_dtype=torch.float32,
                                round_p=round_p).double()
        d = (lg[:, torch.as_tensor(cols)] - ref).abs()
        toks = [int(t) for t in orc.greedy_argmax(lg)]
        return {"rms": float((d * d).mean().sqrt()), "max": float(d.max()),
                "fraction_within_2e-2": float((d <= 2e-2).double().mean()),
                "rows_with_a_different_argmax": int(sum(a != b for a, b in zip(toks, gold["out_tokens"])))}

    plain = one(False, 128)
    rp = [one(True, 128), one(True, 64)]
    return {"_what": "float32-accumulation checker minus float64 checker at the stored columns; 'with_p_rounding': the "
                     "same with the softmax weights rounded to bf16 before P V (prompt cut into windows of 128 and of 64)",
            **plain, "with_p_rounding": rp,
            "model_rms": sum(x["rms"] for x in rp) / len(rp), "model_max": sum(x["max"] for x in rp) / len(rp)}


def main():
    t0 = time.time()
    if "--self-noise-only" in sys.argv:
        shape, prompt, cols = c2_inputs()
        cfg = orc.OracleConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                               shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps)
        gold = json.load(open(OUT))
        gold["self_noise"] = self_noise(gold, cfg, wl.make_weights(shape, seed=SEED), prompt, cols)
        json.dump(gold, open(OUT, "w"))
        print(gold["self_noise"], f"{time.time() - t0:.0f}s", flush=True)
        return
    shape, prompt, cols = c2_inputs()
    cfg = orc.OracleConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                           shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps)
    w = wl.make_weights(shape, seed=SEED)
    print(f"weights {time.time() - t0:.0f}s", flush=True)
    kv = orc.OracleKV(cfg, PROMPT_LEN + WINDOW)
    logits = orc.forward_window(cfg, w, kv, 0, prompt)                       # float64 prefill
    first = int(orc.greedy_argmax(logits[-1:])[0])
    del logits
    print(f"prefill {time.time() - t0:.0f}s first={first}", flush=True)
    # greedy continuation: one token at a time, float32 accumulation on pre-converted weights
    # (it only proposes candidates; the float64 pass below is what is stored)
    w32 = {k: w[k].float() for k in ("embed", "final_norm", "lm_head")}
    w32["layers"] = [{k: v.float() for k, v in lw.items()} for lw in w["layers"]]
    scratch = orc.OracleKV(cfg, kv.capacity)
    scratch.k.copy_(kv.k)
    scratch.v.copy_(kv.v)
    chain, tok = [], first
    for i in range(WINDOW - 1):
        lg = orc.forward_window(cfg, w32, scratch, PROMPT_LEN + i, [tok], acc_dtype=torch.float32)
        tok = int(orc.greedy_argmax(lg)[0])
        chain.append(tok)
        print(f"chain {i} {tok} {time.time() - t0:.0f}s", flush=True)
    del w32, scratch
    base = np.array([[first] + chain], dtype=np.int32)
    cand = wl.replace_candidates(wl.rng_for(SEED, 2, 2), base, RATE, shape.vocab)[0]
    out_tokens, out_logits = orc.verify_window(cfg, w, [kv], [PROMPT_LEN], [cand])
    lg = out_logits[0]
    top = torch.topk(lg, 2, dim=-1)
    committed, ctoks, rolled = orc.commit_rollback(cand, out_tokens[0], WINDOW)
    gold = {
        "_what": "float64 checker results for the 8B-shape, 1 sequence, 512-token prompt, window 32 configuration",
        "_made_by": "tests/golden/make_c2_golden.py (calls only oracle/ and the seeded input generator)",
        "seed": SEED, "prompt_len": PROMPT_LEN, "window": WINDOW, "rate": RATE,
        "first_token": first, "greedy_chain": chain, "candidates": [int(t) for t in cand],
        "out_tokens": out_tokens[0], "committed": committed, "committed_tokens": ctoks, "rolled_back": rolled,
        "top2_ids": top.indices.tolist(), "top2_values": [[round(float(v), 7) for v in r] for r in top.values],
        "logit_abs_max": float(lg.abs().max()), "logit_std": float(lg.std()),
        "columns": cols.tolist(),
        "logits_at_columns": [[round(float(v), 7) for v in r] for r in lg[:, torch.as_tensor(cols)]],
        "kv_samples": {
            "_index": "[layer][window row][kv head 0 and 7][features 0..7]",
            "layers": [0, 15, 31],
            "k": [[[[round(float(x), 7) for x in kv.k[l, PROMPT_LEN + i, h, :8]] for h in (0, 7)]
                   for i in range(WINDOW)] for l in (0, 15, 31)],
            "v": [[[[round(float(x), 7) for x in kv.v[l, PROMPT_LEN + i, h, :8]] for h in (0, 7)]
                   for i in range(WINDOW)] for l in (0, 15, 31)],
        },
    }
    gold["self_noise"] = self_noise(gold, cfg, w, prompt, cols)
    with open(OUT, "w") as f:
        json.dump(gold, f)
    print(f"wrote {OUT} in {time.time() - t0:.0f}s; committed {committed}", flush=True)


if __name__ == "__main__":
    main()
