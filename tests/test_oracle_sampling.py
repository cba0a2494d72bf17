"""Pins for the checker's seeded sampler (paper section 4.4 "Sampling"): the hash against the
published splitmix64 sequence, the Gumbel-max rule against the softmax distribution it must
reproduce, determinism in the key, and the greedy limit."""
import numpy as np
import torch

from helpers import orc


def test_mix64_reproduces_the_splitmix64_sequence():
    # first outputs of the reference splitmix64 generator seeded with 0 (state advances by the golden-ratio
    # increment; output k is the mixing function of k increments): mix64(state_before_increment) == output
    gamma = 0x9E3779B97F4A7C15
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F, 0xF88BB8A8724C81EC]
    got = [int(orc.mix64(np.uint64((k * gamma) & ((1 << 64) - 1)))) for k in range(4)]
    assert got == want


def test_noise_is_a_function_of_the_key_only():
    a = orc.gumbel_noise(7, 11, 300, 64)
    assert np.array_equal(a, orc.gumbel_noise(7, 11, 300, 64))
    for other in (orc.gumbel_noise(8, 11, 300, 64), orc.gumbel_noise(7, 12, 300, 64), orc.gumbel_noise(7, 11, 301, 64)):
        assert not np.array_equal(a, other)
    assert np.isfinite(a).all()


def test_uniforms_are_uniform_and_noise_is_gumbel():
    g = np.concatenate([orc.gumbel_noise(1, 2, p, 4096) for p in range(64)])
    u = np.exp(-np.exp(-g))                                   # back to the uniforms
    hist, _ = np.histogram(u, bins=16, range=(0.0, 1.0))
    expect = len(u) / 16
    assert np.abs(hist - expect).max() < 5 * np.sqrt(expect)  # 5 sigma per bin
    # Gumbel(0, 1): mean = Euler-Mascheroni, variance = pi^2 / 6
    assert abs(g.mean() - 0.5772156649) < 5 * np.sqrt(np.pi ** 2 / 6 / len(g))
    assert abs(g.var() - np.pi ** 2 / 6) < 0.05


def test_gumbel_max_samples_from_the_softmax():
    logits = torch.tensor([[2.0, 1.0, 0.0, -1.0, 0.5, 1.5, -3.0, 0.0]], dtype=torch.float64)
    temperature, n = 0.7, 40000
    counts = np.zeros(8)
    for p in range(n):
        tok, _ = orc.sample_tokens(logits, temperature, seed=123, request_id=5, positions=[p])
        counts[int(tok[0])] += 1
    prob = torch.softmax(logits[0] / temperature, dim=0).numpy()
    sigma = np.sqrt(n * prob * (1 - prob))
    assert (np.abs(counts - n * prob) < 4.5 * sigma).all(), (counts, n * prob)


def test_greedy_limit_and_tie_break():
    logits = torch.tensor([[0.1, 3.0, 3.0, -1.0]], dtype=torch.float64)
    tok, noisy = orc.sample_tokens(logits, 0.0, seed=1, request_id=1, positions=[0])
    assert int(tok[0]) == 1 and noisy is None                 # lowest index among equal maxima
    tok, _ = orc.sample_tokens(torch.tensor([[0.0, 5.0, 1.0]], dtype=torch.float64), 1e-4, 1, 1, [9])
    assert int(tok[0]) == 1                                   # a tiny temperature is the arg-max
