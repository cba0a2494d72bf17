"""Glue shared by the tests: turns a workload ModelShape into the checker's
config, runs the checker's prefill / greedy decode, and small utilities."""
from __future__ import annotations

import os
import sys
from typing import List

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import llm42_oracle as orc  # noqa: E402
from paper_2601_17768_amd import workloads as wl  # noqa: E402


def oracle_cfg(shape: wl.ModelShape) -> orc.OracleConfig:
    return orc.OracleConfig(n_layers=shape.n_layers, d_model=shape.d_model, n_q_heads=shape.n_q_heads,
                            n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ffn=shape.d_ffn,
                            vocab=shape.vocab, rope_theta=shape.rope_theta, rms_eps=shape.rms_eps)


def randomize_gains(weights: dict, seed: int = 7) -> dict:
    """Replace the unit RMSNorm gains by bf16 values around 1 so that a dropped
    or misplaced gain shows up."""
    g = torch.Generator().manual_seed(seed)
    d = weights["final_norm"].numel()
    mk = lambda: (1.0 + 0.25 * torch.randn(d, generator=g)).to(torch.bfloat16)
    for lw in weights["layers"]:
        lw["attn_norm"] = mk()
        lw["ffn_norm"] = mk()
    weights["final_norm"] = mk()
    return weights


def oracle_prefill(cfg, weights, kv, prompt, **kw) -> int:
    """Teacher-forced pass over the prompt from an empty cache; returns the first
    output token (the consistent token T_0 of the paper's DVR figure)."""
    logits = orc.forward_window(cfg, weights, kv, 0, list(prompt), **kw)
    return int(orc.greedy_argmax(logits[-1:])[0])


def oracle_greedy_decode(cfg, weights, kv, seq_len: int, last_token: int, steps: int, **kw) -> List[int]:
    """Plain one-token-at-a-time greedy decoding from a consistent state."""
    out, tok, L = [], int(last_token), int(seq_len)
    for _ in range(steps):
        logits = orc.forward_window(cfg, weights, kv, L, [tok], **kw)
        tok = int(orc.greedy_argmax(logits)[0])
        out.append(tok)
        L += 1
    return out
