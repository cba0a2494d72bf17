"""Host-side pieces of the grouped-verification sweep, pinned to numbers the paper prints: the log-normal
length shapes against the means and medians of its dataset table (section 5, "Workloads"), and the
recompute model against the recompute cost it reports for ungrouped windows (section 4.3)."""
import json
import os

import numpy as np

from helpers import wl
from paper_2601_17768_amd import sweep

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_workload_numbers.json")


def test_length_shapes_reproduce_the_dataset_table():
    table = json.load(open(GOLDEN))["dataset_table"]
    rng = wl.rng_for(7, 1)
    for name, ((mu_in, sd_in), (mu_out, sd_out)) in sweep.LOGNORMAL.items():
        for what, mu, sd in (("input", mu_in, sd_in), ("output", mu_out, sd_out)):
            x = wl.lognormal_lengths(rng, 400000, mu, sd, 1, 10 ** 7).astype(np.float64)
            want = table[name][what]
            assert abs(np.median(x) / want["median"] - 1.0) < 0.03, (name, what, np.median(x))
            assert abs(x.mean() / want["mean"] - 1.0) < 0.06, (name, what, x.mean())


def test_contexts_stay_inside_the_position_range():
    rng = wl.rng_for(7, 2)
    for kind in ("fixed:512", "sharegpt", "arxiv"):
        ctx = sweep.contexts_for(kind, rng, 1000, room=64, max_position=16384)
        assert ctx.dtype == np.int32 and ctx.min() >= 4 and ctx.max() <= 16384 - 64
    assert (sweep.contexts_for("fixed:512", rng, 5, 64, 16384) == 512).all()


def test_recompute_model_matches_the_reported_recompute_cost():
    paper = json.load(open(GOLDEN))["ungrouped_recompute_percent"]
    q = 0.0045                                          # the sweep's default
    for window, percent in paper.items():
        w = int(window)
        e = sweep.expected_committed(w, q)
        assert abs(e - (1.0 - (1.0 - q) ** w) / q) < 1e-9          # closed form of the geometric sum
        model = 100.0 * (1.0 - e / w)
        # the two small windows fix q; at 256 the model is within 6 points of the measurement
        assert abs(model - percent) < (0.4 if w <= 32 else 6.0), (w, model, percent)
    assert sweep.expected_committed(1, 0.3) == 1.0      # a window of one input always commits its one output
    assert abs(sweep.expected_committed(8, 0.0) - 8.0) < 1e-12
