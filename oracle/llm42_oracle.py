"""CPU oracle for the LLM-42 verifier hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition of what the verifier computes.  It is
imported by tests, by the smoke check and by the CPU-baseline leg of the
benchmark, and by nothing else; the product (the HIP library and its Python
binding) never imports it and it never imports the product.  It shares no code,
tables or helpers with the HIP path.

What it defines (paper sections in brackets):

* the verifier forward [§4.1 "Leveraging O2", §4.2]: a window of T inputs
  (one consistent token followed by T-1 candidates) is replayed through a
  decoder-only transformer in one causal pass, producing T output tokens and
  overwriting the window's KV-cache entries [§4.2 "Making KV cache consistent"];
* the sampler [§4.4 "Sampling"]: arg-max of the logits, lowest index among
  equal maxima; for temperature > 0 the logits are first perturbed by Gumbel
  noise that is a hash of (seed, request, position, vocabulary entry);
* the commit / rollback rule [§4.2 Case-1, Case-2, "Guaranteed forward
  progress"]: accept the longest prefix of candidates that the verifier
  reproduces, plus the verifier's own token right after it, and truncate the
  KV cache there.

The paper fixes none of the model's arithmetic (it names the model only:
Llama-3.1-8B, 32 layers, 32 query heads, 8 KV heads [§5 "Models and
environment"]); the decoder block below is the standard pre-norm Llama block
(RMSNorm, rotary embedding with the rotate-half pairing, grouped-query causal
attention, SwiGLU feed-forward) that this model uses.

Arithmetic: every floating-point operation is carried out in `acc_dtype`
(float64 by default; float32 is accepted for speed on big shapes).  Weights are
bf16 values.  When `round_points` is true the activations that the model keeps
in bf16 are rounded to bf16 (round-to-nearest-even) at these points and nowhere
else:
    RMSNorm output;  q and k after the rotary embedding;  v;
    attention output;  SwiGLU output
(the operands of the matrix products, which the device feeds to bf16 matrix
units).  The residual stream and the logits are never rounded: the device keeps
them in fp32.  Rounding the residual stream to bf16 as well was tried and
rejected: two correct evaluations that differ only in summation order then
drift apart by more than the logit tolerance after 32 layers.  (That choice was
made together with the first device kernel, which keeps the residual stream in
fp32: here the checker's contract followed the device's, the wider of the two
options; the paper fixes neither.)  With `round_points` false the whole forward is the
textbook real-number definition evaluated in `acc_dtype`; that mode is what the
pins against an independent library implementation and a brute-force
implementation use.

Pins live in tests/test_oracle_*.py (commit rule against the paper's worked
figure, arg-max ties, closed forms, a library Llama implementation, a
loop-level brute force, prefix purity, stream invariance of the full
decode-verify-rollback loop).
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence, Tuple

import torch


# --------------------------------------------------------------------------
# configuration and state
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class OracleConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float
    rms_eps: float


class OracleKV:
    """Per-sequence KV cache of the oracle: one [capacity, n_kv_heads, head_dim]
    tensor of K and of V per layer, holding bf16-representable values stored in
    float64.  Entries at or beyond the sequence's committed length are garbage by
    definition [§4.2 Case-2: the cache is truncated at the commit point]."""

    def __init__(self, cfg: OracleConfig, capacity: int):
        shape = (cfg.n_layers, capacity, cfg.n_kv_heads, cfg.head_dim)
        self.k = torch.zeros(shape, dtype=torch.float64)
        self.v = torch.zeros(shape, dtype=torch.float64)
        self.capacity = capacity


# --------------------------------------------------------------------------
# scalar building blocks
# --------------------------------------------------------------------------
def bf16_round(x: torch.Tensor) -> torch.Tensor:
    """Round to the nearest bf16 value, ties to even, returned in x's dtype.

    Done on the float32 bit pattern: add 0x7FFF plus the lowest kept bit, then
    clear the 16 dropped bits.  A float64 input is first rounded to float32;
    the double rounding can differ from a single rounding only when the value
    lies within 2^-29 relative of a bf16 tie, which is ignored here."""
    x32 = x.to(torch.float32).contiguous()
    bits = x32.view(torch.int32)
    keep_lsb = (bits >> 16) & 1
    rounded = (bits + 0x7FFF + keep_lsb) & ~0xFFFF
    return rounded.view(torch.float32).to(x.dtype)


def _maybe_round(x: torch.Tensor, round_points: bool) -> torch.Tensor:
    return bf16_round(x) if round_points else x


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """y_j = x_j / sqrt(mean_j(x_j^2) + eps) * gain_j, row-wise over the last dim."""
    mean_sq = (x * x).sum(dim=-1, keepdim=True) / x.shape[-1]
    return x / torch.sqrt(mean_sq + eps) * gain


def rope_angles(positions: torch.Tensor, head_dim: int, theta: float,
                dtype: torch.dtype) -> Tuple[torch.Tensor, torch.Tensor]:
    """cos and sin of position * theta^(-2j/head_dim), j = 0 .. head_dim/2 - 1.
    Evaluated in float64 and cast to `dtype`.  Shape [len(positions), head_dim/2]."""
    j = torch.arange(head_dim // 2, dtype=torch.float64)
    inv_freq = torch.pow(torch.tensor(float(theta), dtype=torch.float64), -2.0 * j / head_dim)
    ang = positions.to(torch.float64)[:, None] * inv_freq[None, :]
    return torch.cos(ang).to(dtype), torch.sin(ang).to(dtype)


def apply_rope(x: torch.Tensor, cos: torch.Tensor, sin: torch.Tensor) -> torch.Tensor:
    """Rotary embedding, rotate-half pairing: element j is paired with j + head_dim/2.
    x: [rows, heads, head_dim]; cos, sin: [rows, head_dim/2]."""
    half = x.shape[-1] // 2
    lo, hi = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return torch.cat([lo * c - hi * s, hi * c + lo * s], dim=-1)


def silu(z: torch.Tensor) -> torch.Tensor:
    return z / (1.0 + torch.exp(-z))


def greedy_argmax(logits: torch.Tensor) -> torch.Tensor:
    """Index of the maximum along the last dim; among equal maxima the lowest
    index [§4.4 "Sampling"].  Written without a library arg-max: find the maximum,
    then the smallest index that attains it."""
    vmax = logits.max(dim=-1, keepdim=True).values
    n = logits.shape[-1]
    idx = torch.arange(n, dtype=torch.int64).expand_as(logits)
    return torch.where(logits == vmax, idx, torch.full_like(idx, n)).min(dim=-1).values


# --------------------------------------------------------------------------
# seeded stochastic sampling [§4.4 "Sampling"]
# --------------------------------------------------------------------------
# The paper's sampler for temperature > 0 perturbs the logits with Gumbel noise that is a pure
# function of a seed and of what is being sampled, and takes the arg-max; the same input and seed
# always give the same token.  The paper does not give the hash; the reading taken here: the noise
# of vocabulary entry v for the token that follows absolute position p of request r is
#     u = (2 * (h >> 41) + 1) / 2^24  with  h = mix(mix(mix(seed ^ mix(r)) ^ p) ^ v),
#     g = -log(-log(u)),
# `mix` being the output function of the splitmix64 generator applied to its argument as state
# (add the golden-ratio increment, two xor-shift-multiply rounds, a final xor-shift), all in
# 64-bit unsigned arithmetic.  The token is argmax_v(logit_v / temperature + g_v), lowest index
# among equal maxima.  Keying by the absolute position (not by the index inside a window) keeps
# the sample independent of how positions are cut into windows.
_M64 = (1 << 64) - 1


def mix64(z):
    """splitmix64 output function on numpy uint64 (wrapping arithmetic)."""
    import numpy as np
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = z + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def gumbel_noise(seed: int, request_id: int, position: int, vocab: int):
    """float64 Gumbel noise for every vocabulary entry of one (request, position)."""
    import numpy as np
    k1 = mix64(np.uint64(seed & _M64) ^ mix64(np.uint64(request_id & _M64)))
    k2 = mix64(k1 ^ np.uint64(position))
    h = mix64(k2 ^ np.arange(vocab, dtype=np.uint64))
    u = (2.0 * (h >> np.uint64(41)).astype(np.float64) + 1.0) / float(1 << 24)
    return -np.log(-np.log(u))


def sample_tokens(logits: torch.Tensor, temperature: float, seed: int, request_id: int,
                  positions: Sequence[int]):
    """One token per row of `logits` ([rows, vocab]); row i belongs to absolute position positions[i].
    temperature == 0 is the greedy sampler.  Returns (tokens, perturbed logits or None)."""
    if temperature == 0:
        return greedy_argmax(logits), None
    import numpy as np
    noisy = torch.empty_like(logits, dtype=torch.float64)
    for i, p in enumerate(positions):
        g = gumbel_noise(seed, request_id, int(p), logits.shape[-1])
        noisy[i] = logits[i].double() / float(temperature) + torch.from_numpy(g)
    return greedy_argmax(noisy), noisy


# --------------------------------------------------------------------------
# verifier forward
# --------------------------------------------------------------------------
def forward_window(cfg: OracleConfig, weights: dict, kv: OracleKV, seq_len: int,
                   tokens: Sequence[int], *, round_points: bool = True,
                   acc_dtype: torch.dtype = torch.float64, round_p: bool = False) -> torch.Tensor:
    """Replay `tokens` (n inputs) of ONE sequence whose first `seq_len` cache
    entries are consistent.  Input i sits at absolute position seq_len + i.
    Writes K and V of every input into cache slots seq_len .. seq_len+n-1 (always,
    whatever was there before [§4.2 "Making KV cache consistent"]) and returns the
    logits [n, vocab] in acc_dtype.  Row i attends to slots 0 .. seq_len+i.

    round_p (off in the definition; used only to measure what one more rounding
    point costs): the unnormalised softmax weights exp(s - max) are rounded to bf16
    before they multiply V, while the denominator sums the unrounded weights - the
    form a bf16 matrix unit needs for the second product of attention."""
    n = len(tokens)
    L = int(seq_len)
    assert n >= 1 and L >= 0 and L + n <= kv.capacity
    f = acc_dtype
    H, G, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    group = H // G
    ids = torch.as_tensor(list(tokens), dtype=torch.int64)
    pos = torch.arange(L, L + n)
    cos, sin = rope_angles(pos, hd, cfg.rope_theta, f)

    r = weights["embed"][ids].to(f)                      # residual stream [n, d]
    for li, lw in enumerate(weights["layers"]):
        y = _maybe_round(rmsnorm(r, lw["attn_norm"].to(f), cfg.rms_eps), round_points)
        q = (y @ lw["wq"].to(f).T).view(n, H, hd)
        k = (y @ lw["wk"].to(f).T).view(n, G, hd)
        v = (y @ lw["wv"].to(f).T).view(n, G, hd)
        q = _maybe_round(apply_rope(q, cos, sin), round_points)
        k = _maybe_round(apply_rope(k, cos, sin), round_points)
        v = _maybe_round(v, round_points)
        kv.k[li, L:L + n] = k.to(torch.float64)
        kv.v[li, L:L + n] = v.to(torch.float64)

        keys = kv.k[li, :L + n].to(f)                    # [L+n, G, hd]
        vals = kv.v[li, :L + n].to(f)
        attn = torch.empty(n, H, hd, dtype=f)
        key_pos = torch.arange(L + n)
        causal = key_pos[None, :] <= pos[:, None]        # [n, L+n]
        for h in range(H):
            g = h // group
            s = (q[:, h, :] @ keys[:, g, :].T) / math.sqrt(hd)      # [n, L+n]
            s = torch.where(causal, s, torch.full_like(s, -math.inf))
            p = torch.exp(s - s.max(dim=-1, keepdim=True).values)
            if round_p:
                attn[:, h, :] = (bf16_round(p) @ vals[:, g, :]) / p.sum(dim=-1, keepdim=True)
            else:
                p = p / p.sum(dim=-1, keepdim=True)
                attn[:, h, :] = p @ vals[:, g, :]
        attn = _maybe_round(attn.reshape(n, H * hd), round_points)
        r = r + attn @ lw["wo"].to(f).T

        y = _maybe_round(rmsnorm(r, lw["ffn_norm"].to(f), cfg.rms_eps), round_points)
        gate = y @ lw["w_gate"].to(f).T
        up = y @ lw["w_up"].to(f).T
        hidden = _maybe_round(silu(gate) * up, round_points)
        r = r + hidden @ lw["w_down"].to(f).T

    y = _maybe_round(rmsnorm(r, weights["final_norm"].to(f), cfg.rms_eps), round_points)
    return y @ weights["lm_head"].to(f).T


# --------------------------------------------------------------------------
# commit / rollback
# --------------------------------------------------------------------------
def commit_rollback(inputs: Sequence[int], outputs: Sequence[int], n_valid: int
                    ) -> Tuple[int, List[int], int]:
    """The accept rule for one sequence [§4.2 Case-1 / Case-2].

    inputs[0] is the consistent token, inputs[1:n_valid] the candidates;
    outputs[i] is the verifier's token after input i.  Candidate inputs[i+1] is
    accepted while it equals outputs[i].  With m accepted candidates the committed
    tokens are outputs[0..m] (m reproduced candidates and the verifier's token
    after the last of them), so committed = m + 1 >= 1 ["Guaranteed forward
    progress"], the rejected candidates number n_valid - 1 - m, and the cache
    keeps the m + 1 inputs that were consistent: new length = old length + m + 1.
    Returns (committed, committed_tokens, rolled_back)."""
    m = 0
    while m < n_valid - 1 and int(inputs[m + 1]) == int(outputs[m]):
        m += 1
    committed = m + 1
    return committed, [int(t) for t in outputs[:committed]], n_valid - 1 - m


def verify_window(cfg: OracleConfig, weights: dict, caches: List[OracleKV],
                  seq_lens: Sequence[int], candidates: Sequence[Sequence[int]],
                  n_valid: Optional[Sequence[int]] = None, *, round_points: bool = True,
                  acc_dtype: torch.dtype = torch.float64, round_p: bool = False
                  ) -> Tuple[List[List[int]], List[torch.Tensor]]:
    """Verifier pass over a group of sequences [§4.3]: every sequence is replayed
    on its own (token positions of different sequences share no data [§3, O3]).
    candidates[s] has `window` entries; only the first n_valid[s] are inputs, the
    rest is padding that is not computed [§4.1: padded positions carry no result].
    Returns per sequence the output tokens (length n_valid[s]) and the logits."""
    out_tokens, out_logits = [], []
    for s, cand in enumerate(candidates):
        n = len(cand) if n_valid is None else int(n_valid[s])
        logits = forward_window(cfg, weights, caches[s], int(seq_lens[s]), list(cand[:n]),
                                round_points=round_points, acc_dtype=acc_dtype, round_p=round_p)
        out_logits.append(logits)
        out_tokens.append([int(t) for t in greedy_argmax(logits)])
    return out_tokens, out_logits


def top2_margin(logits: torch.Tensor) -> torch.Tensor:
    """Per row: largest logit minus second largest (0 for an exact tie)."""
    top = torch.topk(logits, 2, dim=-1).values
    return top[..., 0] - top[..., 1]
