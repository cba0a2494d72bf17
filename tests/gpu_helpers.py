"""Helpers for the GPU parity tests: build the same scenario for the checker and
for the library, move KV contents between the two layouts, compare."""
from __future__ import annotations

import numpy as np
import torch

from helpers import orc, wl, oracle_cfg, oracle_prefill, oracle_greedy_decode
from paper_2601_17768_amd import kv_layout
from paper_2601_17768_amd.session import VerifierSession

ABS_TOL = 2e-2      # spec tolerance on logits: max abs error ...
REL_TOL = 1e-2      # ... and max error relative to the largest logit magnitude


def assert_logits_close(gpu: torch.Tensor, ref: torch.Tensor, what: str = ""):
    """North-star logit tolerance: max |gpu - ref| <= ABS_TOL and <= REL_TOL * max |ref|.
    Used where the logit scale is small enough for it to be meaningful (the small
    configuration: logit std 0.32).  Returns (max abs error, rms error)."""
    g = gpu.detach().cpu().double()
    r = ref.double()
    assert torch.isfinite(g).all(), f"{what}: non-finite GPU logits"
    diff = (g - r).abs()
    err, rms, scale = float(diff.max()), float((diff * diff).mean().sqrt()), float(r.abs().max())
    print(f"{what}: max abs err {err:.3e}, rms {rms:.3e}, logit scale {scale:.2f}, std {float(r.std()):.3f}", flush=True)
    assert err <= ABS_TOL, f"{what}: max abs error {err:.3e} > {ABS_TOL}"
    assert err <= REL_TOL * scale, f"{what}: relative error {err / scale:.3e} > {REL_TOL}"
    return err, rms


NOISE_FACTOR = 1.5   # GPU error allowed relative to the checker-only noise model (measured: 0.9 .. 1.2)


def assert_logits_within_noise(gpu: torch.Tensor, ref: torch.Tensor, noise_rms: float, noise_max: float,
                               what: str = ""):
    """Logit tolerance at the 8B model's widths (logit std 1.3, |logit| up to 7).

    There the benchmark spec's bounds (2e-2 absolute, 1e-2 of the largest logit) cannot hold
    for ANY two correct evaluations with bf16 matrix operands, the checker against itself
    included: each of the model's bf16 rounding points turns a last-bit difference in
    summation order into a one-ulp (0.4 %) difference, and after a few layers the two
    evaluations are decorrelated at that level.  Measured with the checker alone at these widths
    (float32 against float64 accumulation, same inputs): one layer rms 3.9e-3 / max 2.2e-2, two
    layers 6.2e-3 / 3.5e-2, all 32 layers at context 512 rms 2.6e-2 / max 9.4e-2.  A bf16 matrix
    unit adds one rounding point to the definition - the softmax weights are rounded before they
    multiply V - and that alone moves the checker by rms 6.8e-3 / max 3.7e-2 at one layer.
    The tolerance is therefore the checker's own noise on the same inputs with both effects in
    (noise_rms, noise_max: float32 accumulation and rounded softmax weights against the float64
    definition): rms error <= 1.5 noise_rms, max error <= 1.5 noise_max, and the error must
    look like noise - no bias (|mean| <= noise_rms/4), no scale error (|slope against the
    reference| <= 5e-3), correlation >= 0.998.  A structural mistake (wrong index, sign, scale,
    missing term) gives errors of the order of the logit std, 30 to 100 times the noise.
    Returns (max abs error, rms error)."""
    g = gpu.detach().cpu().double()
    r = ref.double()
    assert torch.isfinite(g).all(), f"{what}: non-finite GPU logits"
    e = (g - r).flatten()
    err, rms = float(e.abs().max()), float((e * e).mean().sqrt())
    rc = r.flatten() - r.mean()
    slope = float((e * rc).sum() / (rc * rc).sum())
    corr = float(torch.corrcoef(torch.stack([g.flatten(), r.flatten()]))[0, 1])
    frac = float((e.abs() <= ABS_TOL).double().mean())
    print(f"{what}: max {err:.3e} = {err / noise_max:.2f} x noise, rms {rms:.3e} = {rms / noise_rms:.2f} x noise, "
          f"within-2e-2 {frac:.4f} mean {float(e.mean()):.2e} slope {slope:.2e} corr {corr:.6f} std {float(r.std()):.3f} "
          f"max/scale {err / float(r.abs().max()):.2e}", flush=True)
    assert rms <= NOISE_FACTOR * noise_rms, f"{what}: rms error {rms:.3e} > {NOISE_FACTOR} x {noise_rms:.3e}"
    assert err <= NOISE_FACTOR * noise_max, f"{what}: max error {err:.3e} > {NOISE_FACTOR} x {noise_max:.3e}"
    assert abs(float(e.mean())) <= noise_rms / 4, f"{what}: biased error {float(e.mean()):.3e}"
    assert abs(slope) <= 5e-3, f"{what}: error scales with the logit, slope {slope:.3e}"
    assert corr >= 0.998, f"{what}: correlation {corr:.6f}"
    return err, rms


def checker_noise(cfg, weights, prefix_k, prefix_v, L, tokens, ref_logits):
    """The checker's own noise on one window: float32 accumulation and bf16-rounded softmax weights against the
    float64 definition (ref_logits), on the same cached prefix and inputs.  Returns the |difference| tensor."""
    n = len(tokens)
    kv = orc.OracleKV(cfg, L + n)
    kv.k[:, :L] = prefix_k[:, :L]
    kv.v[:, :L] = prefix_v[:, :L]
    lg = orc.forward_window(cfg, weights, kv, L, tokens, acc_dtype=torch.float32, round_p=True).double()
    return (lg - ref_logits.double()).abs()


def assert_tokens_match_where_decidable(gpu_tokens, gpu_logits, ref_tokens, ref_logits, what=""):
    """Arg-max must agree on every row whose top-1/top-2 margin in the checker exceeds
    twice that row's largest logit error (then no reordering of the top is possible).
    Returns the number of rows that were exempt."""
    g = gpu_logits.detach().cpu().double()
    r = ref_logits.double()
    row_err = (g - r).abs().max(dim=-1).values
    margin = orc.top2_margin(r)
    exempt = 0
    for i in range(r.shape[0]):
        if float(margin[i]) > 2 * float(row_err[i]):
            assert int(gpu_tokens[i]) == int(ref_tokens[i]), f"{what} row {i}"
        else:
            exempt += 1
    return exempt


def oracle_kv_to_gpu(kv_gpu, block_ids, okv: orc.OracleKV, length: int):
    kv_layout.write_tokens(kv_gpu, block_ids, okv.k[:, :length].to(torch.bfloat16),
                           okv.v[:, :length].to(torch.bfloat16), 0)


def gpu_kv_tokens(kv_gpu, block_ids, length: int, head_dim: int):
    k, v = kv_layout.read_tokens(kv_gpu, block_ids, length, head_dim)
    return k.float().cpu().double(), v.float().cpu().double()


class Scenario:
    """A group of sequences with checker-side state: prompts prefilled by the
    checker, its greedy continuation, and candidates with random replacements."""

    def __init__(self, shape, weights, prompts, window, rate, seed, capacity_extra=0):
        self.shape, self.w, self.window = shape, weights, window
        self.cfg = oracle_cfg(shape)
        self.prompts = prompts
        self.lens = np.array([len(p) for p in prompts], dtype=np.int32)
        self.okv, self.first, self.chain = [], [], []
        for p in prompts:
            kv = orc.OracleKV(self.cfg, len(p) + window + capacity_extra)
            t0 = oracle_prefill(self.cfg, weights, kv, p)
            scratch = orc.OracleKV(self.cfg, kv.capacity)
            scratch.k.copy_(kv.k)
            scratch.v.copy_(kv.v)
            self.okv.append(kv)
            self.first.append(t0)
            self.chain.append(oracle_greedy_decode(self.cfg, weights, scratch, len(p), t0, window - 1))
        base = np.array([[f] + c for f, c in zip(self.first, self.chain)], dtype=np.int32)
        self.candidates = wl.replace_candidates(wl.rng_for(seed, 99), base, rate, shape.vocab)

    def oracle_verify(self, n_valid=None):
        return orc.verify_window(self.cfg, self.w, self.okv, self.lens, self.candidates, n_valid)
