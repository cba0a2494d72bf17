"""Seeded synthetic inputs for the verifier: model shapes, random-init weights,
prompts, length mixes, paged block tables and candidate replacement.

This module produces DATA only.  It contains none of the verifier's arithmetic
and is the one piece of code that both the HIP path's callers and the CPU
checker's callers use, so that both see the same inputs.  Weights come from a
small counter-based C generator (synth_gen.c, built into libllm42_synth.so next
to this file); everything else from numpy's PCG64 generator.

Shapes and distributions stand in for the paper's evaluation setting
(Llama-3.1-8B with 32 layers, 32 query heads and 8 KV heads [§5 "Models and
environment"]; verification windows of 32-64 tokens [Table 1]; groups of
requests verified together [§4.3]); no dataset item is reproduced.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libllm42_synth.so")
_lib = None


def build_generator(force: bool = False) -> str:
    """Compile synth_gen.c with gcc (OpenMP).  Returns the library path."""
    src = os.path.join(_HERE, "synth_gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _generator():
    global _lib
    if _lib is None:
        build_generator()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.llm42_synth_normal_bf16.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                                ctypes.c_float, ctypes.c_void_p]
        lib.llm42_synth_normal_bf16.restype = None
        lib.llm42_synth_uniform_i32.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                                ctypes.c_int32, ctypes.c_void_p]
        lib.llm42_synth_uniform_i32.restype = None
        _lib = lib
    return _lib


# --------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float
    rms_eps: float = 1e-5
    kv_block_size: int = 16

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)

    @property
    def gemm_params(self) -> int:
        """Weights streamed by one pass: every matrix except the embedding table."""
        d, f = self.d_model, self.d_ffn
        qkv = d * (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim
        o = self.n_q_heads * self.head_dim * d
        return self.n_layers * (qkv + o + 3 * d * f) + d * self.vocab

    @property
    def kv_bytes_per_token(self) -> int:
        return self.n_layers * 2 * self.n_kv_heads * self.head_dim * 2


TINY = ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                  d_ffn=688, vocab=1024, rope_theta=1e4)
LLAMA_8B = ModelShape(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                      d_ffn=14336, vocab=128256, rope_theta=5e5)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def normal_bf16(seed: int, stream: int, shape: Sequence[int], std: float = 0.02) -> torch.Tensor:
    """bf16 tensor of N(0, std^2) values; a pure function of (seed, stream, shape)."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.bfloat16)
    _generator().llm42_synth_normal_bf16(seed, stream, n, std, out.data_ptr())
    return out.view(*shape)


def uniform_ids(seed: int, stream: int, n: int, bound: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _generator().llm42_synth_uniform_i32(seed, stream, n, bound, out.ctypes.data)
    return out


def make_weights(shape: ModelShape, seed: int = 42, std: float = 0.02) -> Dict:
    """Random-init weights, bf16, every matrix in [out_features, in_features]
    order.  Matrices ~ N(0, std^2); RMSNorm gains are 1 (a N(0, 0.02^2) gain would
    scale every activation to nothing)."""
    d, hd = shape.d_model, shape.head_dim
    ones = lambda: torch.ones(d, dtype=torch.bfloat16)
    w = {"embed": normal_bf16(seed, 1, (shape.vocab, d), std), "layers": []}
    for li in range(shape.n_layers):
        s = 100 + 10 * li
        w["layers"].append({
            "attn_norm": ones(),
            "wq": normal_bf16(seed, s + 0, (shape.n_q_heads * hd, d), std),
            "wk": normal_bf16(seed, s + 1, (shape.n_kv_heads * hd, d), std),
            "wv": normal_bf16(seed, s + 2, (shape.n_kv_heads * hd, d), std),
            "wo": normal_bf16(seed, s + 3, (d, shape.n_q_heads * hd), std),
            "ffn_norm": ones(),
            "w_gate": normal_bf16(seed, s + 4, (shape.d_ffn, d), std),
            "w_up": normal_bf16(seed, s + 5, (shape.d_ffn, d), std),
            "w_down": normal_bf16(seed, s + 6, (d, shape.d_ffn), std),
        })
    w["final_norm"] = ones()
    w["lm_head"] = normal_bf16(seed, 2, (shape.vocab, d), std)
    return w


# --------------------------------------------------------------------------
# sequences, lengths, paging, candidates
# --------------------------------------------------------------------------
def rng_for(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, *stream]))


def uniform_lengths(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in [lo, hi]."""
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def lognormal_lengths(rng: np.random.Generator, n: int, mu: float, sigma: float,
                      lo: int, hi: int) -> np.ndarray:
    """n integers: round(exp(N(mu, sigma^2))) clipped to [lo, hi]."""
    x = np.exp(rng.normal(mu, sigma, size=n))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def random_tokens(rng: np.random.Generator, n: int, vocab: int) -> np.ndarray:
    return rng.integers(0, vocab, size=n).astype(np.int32)


def replace_candidates(rng: np.random.Generator, window_inputs: np.ndarray, rate: float,
                       vocab: int) -> np.ndarray:
    """window_inputs [..., W]: entry 0 is the consistent token, entries 1.. are
    candidates.  Each candidate is replaced, independently with probability
    `rate`, by a uniform random id (which may happen to equal the original).
    Entry 0 is never touched.  Later candidates keep their original values."""
    x = np.array(window_inputs, dtype=np.int32, copy=True)
    mask = rng.random(size=x.shape) < rate
    mask[..., 0] = False
    repl = rng.integers(0, vocab, size=x.shape).astype(np.int32)
    return np.where(mask, repl, x)


def make_block_table(rng: np.random.Generator, tokens_per_seq: Sequence[int], block_size: int,
                     max_blocks_per_seq: Optional[int] = None, spare_blocks: int = 0):
    """Paged-cache block table.  Sequence s needs ceil(tokens/block_size) blocks;
    physical block ids are a random permutation of the pool so that logically
    adjacent blocks are scattered.  Unused table entries hold -1.
    Returns (table int32 [S, max_blocks_per_seq], num_blocks)."""
    need = [(int(t) + block_size - 1) // block_size for t in tokens_per_seq]
    width = max(need) if max_blocks_per_seq is None else max_blocks_per_seq
    assert width >= max(need)
    num_blocks = sum(need) + spare_blocks
    perm = rng.permutation(num_blocks).astype(np.int32)
    table = np.full((len(need), width), -1, dtype=np.int32)
    at = 0
    for s, nb in enumerate(need):
        table[s, :nb] = perm[at:at + nb]
        at += nb
    return table, num_blocks
