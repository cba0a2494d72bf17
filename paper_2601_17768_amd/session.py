"""Buffer management around the binding: uploads weights, owns the model handle,
the workspace and the output tensors, and forwards to the two hot entry points.
No arithmetic of the verifier happens here."""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _to_device(weights: Dict, device) -> Dict:
    out = {k: weights[k].to(device) for k in ("embed", "final_norm", "lm_head")}
    out["layers"] = [{k: v.to(device) for k, v in lw.items()} for lw in weights["layers"]]
    return out


class VerifierSession:
    def __init__(self, shape, weights: Dict, max_position: int, device: str = "cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("the verifier needs a GPU; there is no CPU path")
        self.shape = shape
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = B.make_config(shape, max_position)
        dev_w = weights if weights["embed"].is_cuda else _to_device(weights, self.device)
        self.model = B.llm42_model_create(self.cfg, dev_w)
        del dev_w
        self._ws = None
        self._ws_key = None

    def close(self):
        if self.model:
            torch.cuda.synchronize()
            B.llm42_model_destroy(self.model)
            self.model = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kv_cache(self, num_blocks: int, fill: float = 0.0) -> torch.Tensor:
        from .kv_layout import alloc_kv
        kv = alloc_kv(self.shape, num_blocks, self.device, fill)
        assert kv.numel() * 2 == B.llm42_kv_bytes(self.model, num_blocks)
        return kv

    def workspace(self, num_seqs: int, window: int, max_context: int) -> torch.Tensor:
        need = B.llm42_workspace_bytes(self.model, num_seqs, window, max_context)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def verify(self, kv: torch.Tensor, block_table: torch.Tensor, seq_lens: torch.Tensor,
               candidates: torch.Tensor, n_valid: Optional[torch.Tensor] = None,
               dump_seq_ids: Optional[torch.Tensor] = None, max_context: Optional[int] = None,
               out_tokens: Optional[torch.Tensor] = None, out_logits: Optional[torch.Tensor] = None,
               seq_status: Optional[torch.Tensor] = None, sampling=None):
        """One llm42_verify_window call (llm42_verify_window_sampled if `sampling`, a binding.Sampling,
        is given).  Returns (out_tokens, seq_status, out_logits)."""
        num_seqs, window = candidates.shape
        if max_context is None:
            max_context = block_table.shape[1] * B.LLM42_KV_BLOCK
        ws = self.workspace(num_seqs, window, max_context)
        if out_tokens is None:
            out_tokens = torch.empty((num_seqs, window), dtype=torch.int32, device=self.device)
        if seq_status is None:
            seq_status = torch.empty(num_seqs, dtype=torch.int32, device=self.device)
        if dump_seq_ids is not None and out_logits is None:
            out_logits = torch.zeros((dump_seq_ids.numel(), window, self.shape.vocab), dtype=torch.float32,
                                     device=self.device)
        B.llm42_verify_window(self.model, kv, kv.shape[2], block_table, seq_lens, candidates, window, n_valid,
                              max_context, out_tokens, ws, seq_status, out_logits, dump_seq_ids, sampling=sampling)
        return out_tokens, seq_status, out_logits

    def commit(self, candidates: torch.Tensor, out_tokens: torch.Tensor, seq_lens: torch.Tensor,
               n_valid: Optional[torch.Tensor] = None):
        """One llm42_commit_rollback call; seq_lens is updated in place.
        Returns (committed_counts, committed_tokens, rolled_back_counts)."""
        num_seqs, window = candidates.shape
        counts = torch.empty(num_seqs, dtype=torch.int32, device=self.device)
        tokens = torch.empty((num_seqs, window), dtype=torch.int32, device=self.device)
        rolled = torch.empty(num_seqs, dtype=torch.int32, device=self.device)
        B.llm42_commit_rollback(candidates, out_tokens, n_valid, seq_lens, counts, tokens, rolled)
        return counts, tokens, rolled

    def prefill(self, kv: torch.Tensor, block_table: torch.Tensor, prompts: Sequence[np.ndarray],
                window: int = 32, cached: Optional[torch.Tensor] = None, sampling=None) -> torch.Tensor:
        """One llm42_prefill call: the prompts are appended behind the `cached` positions (int32 [n_seq] on
        the device; none by default) in passes of `window` rows per sequence.  Returns the first output
        token of each sequence (device, int32).  Raises if a sequence was flagged."""
        n_seq = len(prompts)
        lens = np.array([len(p) for p in prompts], dtype=np.int64)
        offsets = np.zeros(n_seq + 1, dtype=np.int32)
        offsets[1:] = np.cumsum(lens)
        flat = np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]) if lens.sum() else np.zeros(1, np.int32)
        if cached is None:
            cached = torch.zeros(n_seq, dtype=torch.int32, device=self.device)
        max_context = min(block_table.shape[1] * B.LLM42_KV_BLOCK, self.cfg.max_position)
        need = B.llm42_prefill_workspace_bytes(self.model, n_seq, window, max_context)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        first = torch.empty(n_seq, dtype=torch.int32, device=self.device)
        status = torch.empty(n_seq, dtype=torch.int32, device=self.device)
        B.llm42_prefill(self.model, kv, kv.shape[2], block_table, cached, torch.as_tensor(flat, device=self.device),
                        torch.as_tensor(offsets, device=self.device), int(lens.max()), window, max_context, first,
                        self._ws, status, sampling=sampling)
        if int(status.max()) != 0:
            raise RuntimeError(f"prefill: sequence status {status.tolist()}")
        return first

    def prefill_by_windows(self, kv: torch.Tensor, block_table: torch.Tensor, prompts: Sequence[np.ndarray],
                           window: int = 32) -> torch.Tensor:
        """The same prefill driven from the host through llm42_verify_window, one call per window over
        the sequences that still have prompt tokens left (what llm42_prefill must reproduce bit for bit).
        Returns the first output token of each sequence."""
        n_seq = len(prompts)
        lens = np.array([len(p) for p in prompts], dtype=np.int32)
        done = np.zeros(n_seq, dtype=np.int32)
        first = torch.full((n_seq,), -1, dtype=torch.int32, device=self.device)
        max_context = int(lens.max())
        while (done < lens).any():
            cand = np.zeros((n_seq, window), dtype=np.int32)
            nv = np.zeros(n_seq, dtype=np.int32)
            for s in range(n_seq):
                n = int(min(window, lens[s] - done[s]))
                nv[s] = n
                if n > 0:
                    cand[s, :n] = prompts[s][done[s]:done[s] + n]
            active = np.nonzero(nv > 0)[0]
            sel = torch.as_tensor(active, device=self.device)
            out, status, _ = self.verify(kv, block_table[sel].contiguous(),
                                         torch.as_tensor(done[active], device=self.device),
                                         torch.as_tensor(cand[active], device=self.device),
                                         torch.as_tensor(nv[active], device=self.device),
                                         max_context=max_context)
            if int(status.max()) != 0:
                raise RuntimeError(f"prefill: sequence status {status.tolist()}")
            done[active] += nv[active]
            fin = [j for j, s in enumerate(active) if done[s] == lens[s]]
            for j in fin:
                first[active[j]] = out[j, nv[active[j]] - 1]
        return first
