"""Cost of a verifier pass per row over the window x group grid (paper section 4.3: small windows are
memory bound - the weights are streamed for a few rows - and large ones compute bound, so the cost per
verified token falls steeply with the rows of a pass and then flattens): ms per row must not increase with
the number of rows, and the knee must sit near the ridge of the machine (2.5 PFLOP/s over 8 TB/s: about 314
rows share one stream of the weights before arithmetic takes over)."""
import numpy as np
import pytest
import torch

from helpers import wl
from gpu_helpers import VerifierSession
from paper_2601_17768_amd import binding as B
from paper_2601_17768_amd.sweep import _time_graph

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.timeout(600)
def test_ms_per_row_falls_then_flattens_near_the_ridge():
    shape = wl.LLAMA_8B.replace(n_layers=4)
    sess = VerifierSession(shape, wl.make_weights(shape, seed=42), max_position=1024, device=DEV)
    per_row = {}
    for group, window in ((1, 16), (1, 32), (1, 64), (8, 16), (8, 32), (8, 64), (16, 64), (32, 64)):
        rng = wl.rng_for(42, 6, group)
        ctx = np.full(group, 512, dtype=np.int32)
        table, num_blocks = wl.make_block_table(rng, ctx + window, 16, spare_blocks=2)
        bt = torch.as_tensor(table, device=DEV)
        kv = sess.kv_cache(num_blocks)
        kv.normal_(generator=torch.Generator(device=DEV).manual_seed(1))
        lens = torch.as_tensor(ctx, device=DEV)
        cand = torch.as_tensor(wl.random_tokens(rng, group * window, shape.vocab).reshape(group, window).astype(np.int32),
                               device=DEV)
        out = torch.empty((group, window), dtype=torch.int32, device=DEV)
        ws = sess.workspace(group, window, 512 + window)
        ms = min(_time_graph(lambda: B.llm42_verify_window(sess.model, kv, num_blocks, bt, lens, cand, window, None,
                                                           512 + window, out, ws), 10) for _ in range(2))
        per_row[group * window] = ms / (group * window)
        print(f"rows {group * window:5d}: {ms:7.3f} ms per pass, {1e3 * per_row[group * window]:7.2f} us per row", flush=True)
        del kv
    rows = sorted(per_row)
    for a, b in zip(rows, rows[1:]):
        assert per_row[b] <= 1.03 * per_row[a], f"ms per row rises from {a} to {b} rows: {per_row[a]:.5f} -> {per_row[b]:.5f}"
    # steep below the ridge (the weight stream is shared by more rows), flat above it (arithmetic per row is constant)
    assert per_row[32] > 4.0 * per_row[512], (per_row[32], per_row[512])
    assert per_row[512] < 2.0 * per_row[2048], (per_row[512], per_row[2048])
    sess.close()
