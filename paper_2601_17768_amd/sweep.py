"""Grouped-verification sweep (paper section 4.3 and the window / group ablation of section 5.3):
for every (window, group size) of a grid, the measured cost of one verifier pass and of one
fast-path decoding step on seeded synthetic sequences, and from them the cost of the
decode - verify - rollback loop per COMMITTED token under a simple divergence model.

    python -m paper_2601_17768_amd.sweep [--lengths fixed:512|sharegpt|arxiv] [--mismatch 0.0045]
                                         [--windows 16,...,512] [--groups 1,...,32] [--layers 32]

Cost model.  One loop iteration for a group of G sequences with window W runs W-1 fast-path steps
(G rows each) and one verifier pass (G x W rows).  If every candidate independently differs from
the verifier's token with probability q, a window commits on average
E(W) = sum_{j=0}^{W-1} (1-q)^j tokens (the matching prefix plus the verifier's own token) and
discards W - E(W) rows of work: the recomputed fraction is 1 - E/W.  The default q = 0.0045
reproduces the recompute cost the paper reports for ungrouped windows of 16 and 32 inputs (3.4 % and
6.8 %; the model then gives 40 % at 256, the paper measured 46 %).  Per grid point the sweep prints
the verifier's ms per row, the recomputed fraction, the verifier's ms per committed token and the
loop's committed tokens per second, and names the grid point with the highest loop throughput.
One JSON line at the end carries the table.

Context lengths.  `fixed:N` gives every sequence N cached tokens.  `sharegpt` and `arxiv` draw, per
sequence, a prompt length and an output length from log-normal fits to the means / medians the
paper's dataset table lists (ShareGPT prompts mu 4.91 sigma 1.27, outputs mu 4.77 sigma 0.99; ArXiv
prompts mu 8.77 sigma 0.42, outputs mu 5.25 sigma 0.37) and place the sequence at a uniformly drawn
point of its output: the shapes of those workloads, none of their items.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np
import torch

from . import binding as B
from . import workloads as wl
from .session import VerifierSession

LOGNORMAL = {"sharegpt": ((4.91, 1.27), (4.77, 0.99)), "arxiv": ((8.77, 0.42), (5.25, 0.37))}


def expected_committed(window: int, q: float) -> float:
    """Mean number of tokens a window of `window` inputs commits when every candidate independently differs from
    the verifier's token with probability q: the matching prefix plus the verifier's own token."""
    return sum((1.0 - q) ** j for j in range(window))


def contexts_for(kind: str, rng: np.random.Generator, n: int, room: int, max_position: int) -> np.ndarray:
    if kind.startswith("fixed:"):
        return np.full(n, int(kind.split(":")[1]), dtype=np.int32)
    (mu_in, sd_in), (mu_out, sd_out) = LOGNORMAL[kind]
    prompt = wl.lognormal_lengths(rng, n, mu_in, sd_in, 4, max_position)
    out = wl.lognormal_lengths(rng, n, mu_out, sd_out, 1, max_position)
    at = np.floor(rng.random(n) * out).astype(np.int32)          # how far into its output the sequence is
    return np.clip(prompt + at, 4, max_position - room).astype(np.int32)


def _time_graph(step, reps: int) -> float:
    for _ in range(2):
        step()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--lengths", default="fixed:512", help="fixed:N, sharegpt or arxiv")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--mismatch", type=float, default=0.0045, help="probability that a candidate differs from the verifier's token")
    ap.add_argument("--windows", default="16,32,64,128,256,512")
    ap.add_argument("--groups", default="1,2,4,8,16,32")
    ap.add_argument("--max-rows", type=int, default=8192, help="grid points with more rows per pass are skipped")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    windows = [int(x) for x in args.windows.split(",")]
    groups = [int(x) for x in args.groups.split(",")]
    if args.lengths not in LOGNORMAL and not args.lengths.startswith("fixed:"):
        sys.exit("--lengths: fixed:N, sharegpt or arxiv")
    shape = wl.LLAMA_8B.replace(n_layers=args.layers)
    weights = wl.make_weights(shape, seed=42)
    max_position = 16384
    sess = VerifierSession(shape, weights, max_position=max_position, device="cuda:0")
    dev = sess.device
    q = args.mismatch
    table = []
    decode_ms = {}
    for window in windows:
        for group in groups:
            if window * group > args.max_rows:
                continue
            rng = wl.rng_for(42, 6, group)                          # the same sequences for every window
            ctx = contexts_for(args.lengths, rng, group, window, max_position)
            bt_host, num_blocks = wl.make_block_table(rng, ctx + window, 16, spare_blocks=4)
            bt = torch.as_tensor(bt_host, device=dev)
            kv = sess.kv_cache(num_blocks)
            kv.normal_(generator=torch.Generator(device=dev).manual_seed(1))
            lens = torch.as_tensor(ctx, device=dev)
            cand = torch.as_tensor(wl.random_tokens(rng, group * window, shape.vocab).reshape(group, window).astype(np.int32),
                                   device=dev)
            out = torch.empty((group, window), dtype=torch.int32, device=dev)
            max_context = int(ctx.max()) + window
            ws = sess.workspace(group, window, max_context)
            pass_ms = _time_graph(lambda: B.llm42_verify_window(sess.model, kv, num_blocks, bt, lens, cand, window, None,
                                                                max_context, out, ws), args.reps)
            if group not in decode_ms:                              # one fast-path step for the group
                nxt = torch.empty(group, dtype=torch.int32, device=dev)
                tok = cand[:, 0].contiguous()
                ws1 = sess.workspace(group, 1, max_context)
                decode_ms[group] = _time_graph(lambda: B.llm42_decode_step(sess.model, kv, num_blocks, bt, lens, tok,
                                                                           max_context, nxt, ws1), args.reps)
            expect = expected_committed(window, q)
            iteration_ms = (window - 1) * decode_ms[group] + pass_ms
            row = {"window": window, "group": group, "rows": window * group, "context_mean": round(float(ctx.mean()), 1),
                   "pass_ms": round(pass_ms, 4), "ms_per_row": round(pass_ms / (window * group), 5),
                   "decode_step_ms": round(decode_ms[group], 4),
                   "expected_committed": round(expect, 2), "recomputed_fraction": round(1.0 - expect / window, 4),
                   "verify_ms_per_committed_token": round(pass_ms / (group * expect), 5),
                   "loop_tokens_per_s": round(group * expect / iteration_ms * 1e3, 1)}
            table.append(row)
            print(f"window {window:3d} group {group:3d} rows {window * group:5d}: pass {pass_ms:8.3f} ms "
                  f"{row['ms_per_row']:.4f} ms/row | recomputed {100 * row['recomputed_fraction']:5.1f} % | verifier "
                  f"{row['verify_ms_per_committed_token']:.4f} ms per committed token | loop {row['loop_tokens_per_s']:9.1f} tok/s",
                  file=sys.stderr, flush=True)
    best = max(table, key=lambda r: r["loop_tokens_per_s"])
    cheapest = min(table, key=lambda r: r["verify_ms_per_committed_token"])
    sess.close()
    print(json.dumps({"lengths": args.lengths, "n_layers": args.layers, "mismatch": q, "grid": table,
                      "best_loop_throughput": best, "cheapest_verification": cheapest}), flush=True)


if __name__ == "__main__":
    main()
