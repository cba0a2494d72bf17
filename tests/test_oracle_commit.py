"""Pins for the checker's commit/rollback rule and greedy sampler
(paper Section 4.2 Case-1 / Case-2 / forward progress, Section 4.4 Sampling)."""
import json
import os

import numpy as np
import pytest
import torch

from helpers import orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dvr_figure_cases.json")


@pytest.mark.parametrize("idx", [0, 1])
def test_paper_figure_cases(idx):
    case = json.load(open(GOLDEN))["cases"][idx]
    committed, tokens, rolled = orc.commit_rollback(case["inputs"], case["verifier_outputs"], 4)
    assert committed == case["committed"]
    assert tokens == case["committed_tokens"]
    assert rolled == case["rolled_back"]
    # KV truncation point: old length + committed
    assert committed == case["kv_len_increase"]


def test_forward_progress_when_nothing_matches():
    # every candidate wrong: still one new consistent token (the verifier's first output)
    committed, tokens, rolled = orc.commit_rollback([5, 6, 7, 8], [1, 2, 3, 4], 4)
    assert (committed, tokens, rolled) == (1, [1], 3)


def test_window_of_one_has_no_candidates():
    assert orc.commit_rollback([5], [9], 1) == (1, [9], 0)


def test_match_after_a_mismatch_is_not_accepted():
    # candidate 2 is wrong, candidate 3 would match: the prefix rule stops at 2
    committed, tokens, rolled = orc.commit_rollback([0, 1, 99, 3], [1, 2, 3, 4], 4)
    assert (committed, tokens, rolled) == (2, [1, 2], 2)


def test_padding_is_never_compared():
    # n_valid = 3 of a window of 5: entries 3, 4 are padding and would "match"
    committed, tokens, rolled = orc.commit_rollback([0, 1, 2, 3, 4], [1, 2, 3, 4, 5], 3)
    assert (committed, tokens, rolled) == (3, [1, 2, 3], 0)


def test_against_vectorised_brute_force():
    rng = np.random.default_rng(0)
    for _ in range(500):
        W = int(rng.integers(1, 12))
        n = int(rng.integers(1, W + 1))
        x = rng.integers(0, 3, size=W)
        y = rng.integers(0, 3, size=W)
        committed, tokens, rolled = orc.commit_rollback(x, y, n)
        hits = (x[1:n] == y[:n - 1]).astype(int)
        m = int(np.cumprod(hits).sum()) if n > 1 else 0       # leading run of hits
        assert committed == m + 1 and rolled == n - 1 - m
        assert tokens == [int(t) for t in y[:m + 1]]
        assert 1 <= committed <= n and committed + rolled == n


def test_mean_committed_matches_closed_form():
    """Greedy candidates replaced i.i.d. with prob. rate by a uniform id miss with
    rho = rate (1 - 1/V); committed = 1 + leading hits among W-1 candidates, so
    E[committed] = sum_{j<W} (1-rho)^j = (1 - (1-rho)^W) / rho."""
    rng = np.random.default_rng(1)
    W, rate, V, trials = 8, 0.1, 1024, 20000
    chain = np.arange(1, W + 1)                       # verifier outputs y_i = i + 1
    total = 0
    for _ in range(trials):
        x = np.arange(0, W)                           # inputs x_{i+1} = y_i: all hits
        mask = rng.random(W) < rate
        mask[0] = False
        x = np.where(mask, rng.integers(0, V, size=W), x)
        total += orc.commit_rollback(x, chain, W)[0]
    rho = rate * (1 - 1 / V)
    expect = (1 - (1 - rho) ** W) / rho
    assert abs(expect - 5.70) < 0.01                  # value for W=8, rate 0.1
    assert abs(total / trials - expect) < 0.06        # ~4 sigma of the sample mean


def test_argmax_planted_ties_pick_lowest_index():
    x = torch.tensor([[0.0, 3.0, 1.0, 3.0, 3.0], [2.0, 2.0, 2.0, 2.0, 2.0], [-1.0, -5.0, -1.0, -7.0, -9.0]],
                     dtype=torch.float64)
    assert orc.greedy_argmax(x).tolist() == [1, 0, 0]
    # independent of where the maximum sits
    rng = np.random.default_rng(2)
    for _ in range(100):
        v = torch.tensor(rng.integers(0, 4, size=(3, 17)).astype(np.float64))
        got = orc.greedy_argmax(v).tolist()
        for row, g in zip(v.tolist(), got):
            assert g == row.index(max(row))


def test_top2_margin():
    x = torch.tensor([[0.0, 3.0, 1.0, 2.5], [1.0, 1.0, 0.0, 0.0]], dtype=torch.float64)
    assert orc.top2_margin(x).tolist() == [0.5, 0.0]
