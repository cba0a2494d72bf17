"""Grouped-verification sweep (paper section 4.3 and its window / group ablation): verifier cost per
row for every (window, group size) of a grid, on seeded synthetic sequences of one context length,
plus the expected cost per COMMITTED token under a simple divergence model.

    python -m paper_2601_17768_amd.sweep [--context 512] [--layers 32] [--mismatch 0.02]

The verifier streams all weights once per pass, so the cost per row falls with rows = window x
group until the GEMMs turn compute bound; larger windows, however, lose more work per rollback.
With an independent per-candidate mismatch probability q, a window of W inputs commits on average
E = sum_{j=0}^{W-1} (1-q)^j tokens (the matching prefix plus the verifier's own token), so the
verifier time per committed token is  pass time / (group x E).  The sweep prints both and the
grid point that minimises the second.  One JSON line at the end carries the table.
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--context", type=int, default=512)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--mismatch", type=float, default=0.02, help="per-candidate probability that the fast path's token differs")
    ap.add_argument("--windows", default="16,32,64")
    ap.add_argument("--groups", default="1,2,4,8,16,32")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    windows = [int(x) for x in args.windows.split(",")]
    groups = [int(x) for x in args.groups.split(",")]
    shape = wl.LLAMA_8B.replace(n_layers=args.layers)
    weights = wl.make_weights(shape, seed=42)
    sess = VerifierSession(shape, weights, max_position=args.context + 2 * max(windows), device="cuda:0")
    dev = sess.device
    rng = wl.rng_for(42, 6, 1)
    table = []
    for window in windows:
        for group in groups:
            ctx = np.full(group, args.context, dtype=np.int32)
            bt_host, num_blocks = wl.make_block_table(rng, ctx + window, 16, spare_blocks=4)
            bt = torch.as_tensor(bt_host, device=dev)
            kv = sess.kv_cache(num_blocks)
            kv.normal_(generator=torch.Generator(device=dev).manual_seed(1))
            lens = torch.as_tensor(ctx, device=dev)
            cand = torch.as_tensor(wl.random_tokens(rng, group * window, shape.vocab).reshape(group, window).astype(np.int32),
                                   device=dev)
            out = torch.empty((group, window), dtype=torch.int32, device=dev)
            max_context = args.context + window
            ws = sess.workspace(group, window, max_context)

            def step():
                B.llm42_verify_window(sess.model, kv, num_blocks, bt, lens, cand, window, None, max_context, out, ws)

            for _ in range(2):
                step()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.reps):
                graph.replay()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.reps
            q = args.mismatch
            expect = sum((1.0 - q) ** j for j in range(window))
            row = {"window": window, "group": group, "rows": window * group, "pass_ms": round(ms, 4),
                   "ms_per_row": round(ms / (window * group), 5),
                   "ms_per_committed_token": round(ms / (group * expect), 5)}
            table.append(row)
            print(f"window {window:3d} group {group:3d} rows {window * group:5d}: pass {ms:8.3f} ms, "
                  f"{row['ms_per_row']:.4f} ms/row, {row['ms_per_committed_token']:.4f} ms per committed token", file=sys.stderr, flush=True)
    best = min(table, key=lambda r: r["ms_per_committed_token"])
    sess.close()
    print(json.dumps({"context": args.context, "n_layers": args.layers, "mismatch": args.mismatch, "grid": table,
                      "best": best}), flush=True)


if __name__ == "__main__":
    main()
