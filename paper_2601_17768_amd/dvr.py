"""Decode - verify - rollback loop (paper section 4.1-4.2) on top of the library calls.

Host logic only: which call comes next and with which buffers.  Every token is produced by
llm42_decode_step (fast path, reduction order follows the batch), checked by
llm42_verify_window (fixed schedule) and committed by llm42_commit_rollback.

One iteration for a group of sequences with consistent state (L cached positions, last
consistent token t0), window W:
  1. fast path: W-1 greedy steps from t0; their K/V land in cache slots L .. L+W-2
  2. verifier: replay [t0, c1 .. c(W-1)] at positions L .. L+W-1 (overwrites those slots)
  3. commit: longest matching prefix + the verifier's own next token; L grows by that many
The committed stream of a sequence is a function of its own consistent prefix only, so it
does not depend on which other sequences share the group - which is what the tests check.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import torch

from . import binding as B
from .session import VerifierSession


@dataclass
class DvrStats:
    iterations: int = 0
    fast_tokens: int = 0          # candidate tokens produced by the fast path
    verified_rows: int = 0        # rows replayed by the verifier
    committed: int = 0            # tokens committed
    rolled_back: int = 0          # candidates discarded (recomputed later)
    rollbacks: int = 0            # windows with at least one discarded candidate
    per_iteration_committed: List[int] = field(default_factory=list)


def generate(sess: VerifierSession, kv: torch.Tensor, block_table: torch.Tensor, seq_lens: torch.Tensor,
             first_tokens: torch.Tensor, max_new: int, window: int, sampling=None):
    """Runs the loop until every sequence has at least max_new committed tokens.

    seq_lens (int32 [B], device) is advanced in place; first_tokens (int32 [B]) are the consistent
    tokens T_0 whose K/V are not yet cached.  `sampling` (binding.Sampling or None = greedy) is
    used by the fast path and by the verifier alike.  Returns (tokens [B, max_new] on the host, DvrStats).
    The cache must have room for seq_lens + max_new + 2 * window positions per sequence."""
    if window < 2:
        raise ValueError("the loop needs at least one candidate per window")
    dev = sess.device
    n_seq = seq_lens.numel()
    num_blocks = kv.shape[2]
    max_context = block_table.shape[1] * B.LLM42_KV_BLOCK
    ws = sess.workspace(n_seq, window, max_context)
    cand = torch.empty((n_seq, window), dtype=torch.int32, device=dev)
    out = torch.empty((n_seq, window), dtype=torch.int32, device=dev)
    nxt = torch.empty(n_seq, dtype=torch.int32, device=dev)
    counts = torch.empty(n_seq, dtype=torch.int32, device=dev)
    ctoks = torch.empty((n_seq, window), dtype=torch.int32, device=dev)
    rolled = torch.empty(n_seq, dtype=torch.int32, device=dev)
    t0 = first_tokens.to(device=dev, dtype=torch.int32).clone()
    streams: List[List[int]] = [[] for _ in range(n_seq)]
    stats = DvrStats()
    rows = torch.arange(n_seq, device=dev)
    while min(len(s) for s in streams) < max_new:
        # 1. fast path
        cand[:, 0] = t0
        fast_lens = seq_lens.clone()
        cur = t0.clone()
        for i in range(1, window):
            B.llm42_decode_step(sess.model, kv, num_blocks, block_table, fast_lens, cur, max_context, nxt, ws,
                                sampling=sampling)
            cand[:, i] = nxt
            cur = nxt.clone()
            fast_lens += 1
        # 2. verifier, 3. commit
        B.llm42_verify_window(sess.model, kv, num_blocks, block_table, seq_lens, cand, window, None, max_context, out, ws,
                              sampling=sampling)
        B.llm42_commit_rollback(cand, out, None, seq_lens, counts, ctoks, rolled)
        t0 = ctoks[rows, (counts - 1).long()].clone()      # the corrected (or next) token: consistent by construction
        c_host, t_host, r_host = counts.cpu().tolist(), ctoks.cpu().tolist(), rolled.cpu().tolist()
        for s in range(n_seq):
            streams[s].extend(t_host[s][:c_host[s]])
        stats.iterations += 1
        stats.fast_tokens += n_seq * (window - 1)
        stats.verified_rows += n_seq * window
        stats.committed += sum(c_host)
        stats.rolled_back += sum(r_host)
        stats.rollbacks += sum(1 for r in r_host if r > 0)
        stats.per_iteration_committed.append(sum(c_host))
    return torch.tensor([s[:max_new] for s in streams], dtype=torch.int32), stats


def generate_verifier_only(sess: VerifierSession, kv: torch.Tensor, block_table: torch.Tensor,
                           seq_lens: torch.Tensor, first_tokens: torch.Tensor, max_new: int, sampling=None):
    """The reference the loop must reproduce: one token at a time through the verifier alone
    (fixed schedule for every token; what the paper calls running everything deterministically)."""
    dev = sess.device
    n_seq = seq_lens.numel()
    num_blocks = kv.shape[2]
    max_context = block_table.shape[1] * B.LLM42_KV_BLOCK
    ws = sess.workspace(n_seq, 1, max_context)
    cur = first_tokens.to(device=dev, dtype=torch.int32).clone().view(n_seq, 1)
    out = torch.empty((n_seq, 1), dtype=torch.int32, device=dev)
    toks = []
    for _ in range(max_new):
        B.llm42_verify_window(sess.model, kv, num_blocks, block_table, seq_lens, cur, 1, None, max_context, out, ws,
                              sampling=sampling)
        seq_lens += 1
        toks.append(out[:, 0].clone())
        cur = out.clone()
    return torch.stack(toks, dim=1).cpu()
