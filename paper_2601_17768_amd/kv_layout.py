"""Index helpers for the paged KV-cache layout documented in include/llm42.h.

The cache is one bf16 tensor [n_layers, 2, num_blocks, n_kv_heads, 16 * head_dim];
these functions only move values between that layout and plain
[n_layers, tokens, n_kv_heads, head_dim] arrays (pure indexing, no arithmetic).
"""
from __future__ import annotations

import torch


def alloc_kv(shape, num_blocks: int, device, fill: float = 0.0) -> torch.Tensor:
    return torch.full((shape.n_layers, 2, num_blocks, shape.n_kv_heads, 16 * shape.head_dim), fill,
                      dtype=torch.bfloat16, device=device)


def _tiles_to_tokens_k(t: torch.Tensor, hd: int) -> torch.Tensor:
    # [L, nb, H, 16*hd] with K tile order (feature group of 8, token, 8) -> [L, nb*16, H, hd]
    L, nb, H, _ = t.shape
    return t.view(L, nb, H, hd // 8, 16, 8).permute(0, 1, 4, 2, 3, 5).reshape(L, nb * 16, H, hd)


def _tiles_to_tokens_v(t: torch.Tensor, hd: int) -> torch.Tensor:
    # V tile order (feature block of 16, token group of 4, feature, token) -> [L, nb*16, H, hd]
    L, nb, H, _ = t.shape
    return t.view(L, nb, H, hd // 16, 4, 16, 4).permute(0, 1, 4, 6, 2, 3, 5).reshape(L, nb * 16, H, hd)


def _tokens_to_tiles_k(x: torch.Tensor, hd: int) -> torch.Tensor:
    L, T, H, _ = x.shape
    return x.view(L, T // 16, 16, H, hd // 8, 8).permute(0, 1, 3, 4, 2, 5).reshape(L, T // 16, H, 16 * hd)


def _tokens_to_tiles_v(x: torch.Tensor, hd: int) -> torch.Tensor:
    L, T, H, _ = x.shape
    return x.view(L, T // 16, 4, 4, H, hd // 16, 16).permute(0, 1, 4, 5, 2, 6, 3).reshape(L, T // 16, H, 16 * hd)


def read_tokens(kv: torch.Tensor, block_ids: torch.Tensor, length: int, head_dim: int):
    """K and V of positions 0..length-1 of the sequence whose blocks are `block_ids`
    (1-D, in logical order).  Returns two [n_layers, length, n_kv_heads, head_dim] tensors."""
    nb = (length + 15) // 16
    ids = block_ids[:nb].long()
    k = _tiles_to_tokens_k(kv[:, 0, ids], head_dim)[:, :length]
    v = _tiles_to_tokens_v(kv[:, 1, ids], head_dim)[:, :length]
    return k, v


def write_tokens(kv: torch.Tensor, block_ids: torch.Tensor, k: torch.Tensor, v: torch.Tensor, start: int = 0):
    """Store k, v ([n_layers, n, n_kv_heads, head_dim]) at positions start..start+n-1."""
    hd = k.shape[-1]
    n = k.shape[1]
    b0, b1 = start // 16, (start + n + 15) // 16
    ids = block_ids[b0:b1].long()
    cur_k = _tiles_to_tokens_k(kv[:, 0, ids], hd).clone()
    cur_v = _tiles_to_tokens_v(kv[:, 1, ids], hd).clone()
    off = start - b0 * 16
    cur_k[:, off:off + n] = k.to(kv.dtype).to(kv.device)
    cur_v[:, off:off + n] = v.to(kv.dtype).to(kv.device)
    kv[:, 0, ids] = _tokens_to_tiles_k(cur_k, hd)
    kv[:, 1, ids] = _tokens_to_tiles_v(cur_v, hd)
