"""ctypes binding of the verifier library (include/llm42.h).

Argument marshalling only: every function here has the name and meaning of the
C entry point it wraps, takes torch tensors where the C call takes device
pointers, and raises `Llm42Error` on a negative status.  No step of the
verifier runs in Python; if libllm42.so is missing the import of the library
fails loudly - there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libllm42.so")

LLM42_OK, LLM42_EINVAL, LLM42_ESHAPE, LLM42_EWORKSPACE, LLM42_ECAPACITY, LLM42_EHIP = 0, -1, -2, -3, -4, -5
LLM42_KV_BLOCK = 16
LLM42_MAX_WINDOW = 512
LLM42_MAX_ROWS = 65536
LLM42_STATIC_SCRATCH_BYTES = 64 << 20
LLM42_SEQ_OK, LLM42_SEQ_BAD_LENGTH, LLM42_SEQ_BAD_BLOCK, LLM42_SEQ_BAD_TOKEN = 0, 1, 2, 4

EXPORTS = ("llm42_model_create", "llm42_model_destroy", "llm42_kv_bytes", "llm42_workspace_bytes",
           "llm42_verify_window", "llm42_verify_window_static", "llm42_commit_rollback", "llm42_last_error", "llm42_schedule_info",
           "llm42_profile_enable", "llm42_profile_collect", "llm42_measure_verify_window_batch_chosen", "llm42_measure_attention_plan", "llm42_decode_step", "llm42_verify_window_sampled",
           "llm42_decode_step_sampled", "llm42_prefill", "llm42_prefill_workspace_bytes")
KERNEL_CLASSES = ("prepare", "embed", "rmsnorm", "qkv", "attention", "o_proj", "gate_up", "down", "lm_head",
                  "argmax", "commit")


class Llm42Error(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"llm42 status {status}: {message}")
        self.status = status


class Config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("rope_theta", ctypes.c_float), ("rms_eps", ctypes.c_float),
                ("kv_block_size", ctypes.c_int32), ("max_position", ctypes.c_int32)]


class Weights(ctypes.Structure):
    _fields_ = [("embed", ctypes.c_void_p), ("final_norm", ctypes.c_void_p), ("lm_head", ctypes.c_void_p)] + \
               [(n, ctypes.POINTER(ctypes.c_void_p)) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class Sampling(ctypes.Structure):
    _fields_ = [("temperature", ctypes.c_float), ("seed", ctypes.c_uint64), ("request_ids", ctypes.c_void_p)]


def make_sampling(temperature: float, seed: int, request_ids: Optional[torch.Tensor] = None) -> Sampling:
    """request_ids: int64 device tensor [num_seqs] or None (then the index in the call is the id)."""
    return Sampling(float(temperature), int(seed) & ((1 << 64) - 1), _ptr(request_ids, torch.int64))


class KVCache(ctypes.Structure):
    _fields_ = [("kv_base", ctypes.c_void_p), ("num_blocks", ctypes.c_int64), ("block_table", ctypes.c_void_p),
                ("max_blocks_per_seq", ctypes.c_int32)]


_lib = None


def load_library(path: Optional[str] = None):
    """dlopen libllm42.so (built by paper_2601_17768_amd.build) and declare its signatures."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built; run `python -m paper_2601_17768_amd.build`")
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.llm42_model_create.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(Weights), ctypes.POINTER(vp)]
    lib.llm42_model_create.restype = i32
    lib.llm42_model_destroy.argtypes = [vp]
    lib.llm42_model_destroy.restype = None
    lib.llm42_kv_bytes.argtypes = [vp, i64, ctypes.POINTER(ctypes.c_size_t)]
    lib.llm42_kv_bytes.restype = i32
    lib.llm42_workspace_bytes.argtypes = [vp, i32, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.llm42_workspace_bytes.restype = i32
    lib.llm42_verify_window.argtypes = [vp, ctypes.POINTER(KVCache), vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, i32,
                                        vp, ctypes.c_size_t, vp]
    lib.llm42_verify_window.restype = i32
    lib.llm42_verify_window_static.argtypes = [vp, ctypes.POINTER(KVCache), vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, i32, vp]
    lib.llm42_verify_window_static.restype = i32
    lib.llm42_verify_window_sampled.argtypes = lib.llm42_verify_window.argtypes + [ctypes.POINTER(Sampling)]
    lib.llm42_verify_window_sampled.restype = i32
    lib.llm42_decode_step.argtypes = [vp, ctypes.POINTER(KVCache), vp, vp, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.llm42_decode_step.restype = i32
    lib.llm42_decode_step_sampled.argtypes = lib.llm42_decode_step.argtypes + [ctypes.POINTER(Sampling)]
    lib.llm42_decode_step_sampled.restype = i32
    lib.llm42_prefill_workspace_bytes.argtypes = lib.llm42_workspace_bytes.argtypes
    lib.llm42_prefill_workspace_bytes.restype = i32
    lib.llm42_prefill.argtypes = [vp, ctypes.POINTER(KVCache), vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, ctypes.c_size_t,
                                  vp, ctypes.POINTER(Sampling)]
    lib.llm42_prefill.restype = i32
    lib.llm42_commit_rollback.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
    lib.llm42_commit_rollback.restype = i32
    lib.llm42_profile_enable.argtypes = [i32, i32]
    lib.llm42_profile_enable.restype = i32
    lib.llm42_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32), i32,
                                          ctypes.POINTER(i32)]
    lib.llm42_profile_collect.restype = i32
    lib.llm42_measure_verify_window_batch_chosen.argtypes = lib.llm42_verify_window.argtypes
    lib.llm42_measure_verify_window_batch_chosen.restype = i32
    lib.llm42_measure_attention_plan.argtypes = [vp, i32, i32, i32, ctypes.POINTER(i64)]
    lib.llm42_measure_attention_plan.restype = i32
    lib.llm42_last_error.argtypes = []
    lib.llm42_last_error.restype = ctypes.c_char_p
    lib.llm42_schedule_info.argtypes = []
    lib.llm42_schedule_info.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != LLM42_OK:
        raise Llm42Error(status, load_library().llm42_last_error().decode())


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _kv_view(model: int, kv_base: torch.Tensor, num_blocks: int, block_table: torch.Tensor, num_seqs: int) -> KVCache:
    """The C struct for a KV tensor and its block table; refuses a tensor smaller than num_blocks blocks need
    (the library sees a bare pointer and could not tell)."""
    if block_table.dim() != 2 or block_table.shape[0] != num_seqs:
        raise ValueError("block_table must be [num_seqs, max_blocks_per_seq]")
    need = llm42_kv_bytes(model, num_blocks)
    if kv_base.numel() * kv_base.element_size() < need:
        raise ValueError(f"kv_base holds {kv_base.numel() * kv_base.element_size()} bytes, {num_blocks} blocks need {need}")
    return KVCache(_ptr(kv_base), num_blocks, _ptr(block_table, torch.int32), block_table.shape[1])


def make_config(shape, max_position: int) -> Config:
    """`shape` is any object with the model-dimension attributes (e.g. workloads.ModelShape)."""
    return Config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                  shape.vocab, float(shape.rope_theta), float(shape.rms_eps), int(shape.kv_block_size),
                  int(max_position))


def llm42_model_create(cfg: Config, weights: Dict) -> int:
    """weights: {'embed','final_norm','lm_head': tensor, 'layers': [ {name: tensor} ]}, bf16 DEVICE
    tensors in [out_features, in_features] order.  Returns the opaque model handle."""
    lib = load_library()
    n = cfg.n_layers
    w = Weights()
    keep = []
    for name in ("embed", "final_norm", "lm_head"):
        setattr(w, name, _ptr(weights[name], torch.bfloat16))
    for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
        arr = (ctypes.c_void_p * n)(*[_ptr(weights["layers"][l][name], torch.bfloat16) for l in range(n)])
        keep.append(arr)
        setattr(w, name, ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p)))
    torch.cuda.synchronize()                       # the source tensors must be complete
    handle = ctypes.c_void_p()
    _check(lib.llm42_model_create(ctypes.byref(cfg), ctypes.byref(w), ctypes.byref(handle)))
    return handle.value


def llm42_model_destroy(model: int) -> None:
    load_library().llm42_model_destroy(model)


def llm42_kv_bytes(model: int, num_blocks: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().llm42_kv_bytes(model, num_blocks, ctypes.byref(out)))
    return out.value


def llm42_workspace_bytes(model: int, max_seqs: int, window: int, max_context: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().llm42_workspace_bytes(model, max_seqs, window, max_context, ctypes.byref(out)))
    return out.value


def llm42_verify_window(model: int, kv_base: torch.Tensor, num_blocks: int, block_table: torch.Tensor,
                        seq_lens: torch.Tensor, candidates: torch.Tensor, window: int,
                        n_valid: Optional[torch.Tensor], max_context: int, out_tokens: torch.Tensor,
                        workspace: torch.Tensor, seq_status: Optional[torch.Tensor] = None,
                        out_logits: Optional[torch.Tensor] = None, dump_seq_ids: Optional[torch.Tensor] = None,
                        stream=None, sampling: Optional[Sampling] = None, batch_chosen: bool = False) -> None:
    """sampling given: llm42_verify_window_sampled.  batch_chosen (measurement only):
    llm42_measure_verify_window_batch_chosen, the same pass off the fixed schedule."""
    num_seqs = seq_lens.numel()
    if candidates.shape != (num_seqs, window) or out_tokens.shape != (num_seqs, window):
        raise ValueError("candidates / out_tokens must be [num_seqs, window]")
    n_dump = 0 if dump_seq_ids is None else dump_seq_ids.numel()
    if n_dump and (out_logits is None or out_logits.shape[0] != n_dump or out_logits.shape[1] != window):
        raise ValueError("out_logits must be [n_dump, window, vocab]")
    kv = _kv_view(model, kv_base, num_blocks, block_table, num_seqs)
    args = (model, ctypes.byref(kv), _ptr(seq_lens, torch.int32), _ptr(candidates, torch.int32), window,
            _ptr(n_valid, torch.int32), num_seqs, max_context, _ptr(out_tokens, torch.int32),
            _ptr(seq_status, torch.int32), _ptr(out_logits, torch.float32), _ptr(dump_seq_ids, torch.int32), n_dump,
            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if batch_chosen:
        if sampling is not None:
            raise ValueError("the measurement entry has no sampled form")
        _check(load_library().llm42_measure_verify_window_batch_chosen(*args))
    elif sampling is None:
        _check(load_library().llm42_verify_window(*args))
    else:
        _check(load_library().llm42_verify_window_sampled(*args, ctypes.byref(sampling)))


def llm42_verify_window_static(model: int, kv_base: torch.Tensor, num_blocks: int, block_table: torch.Tensor,
                               seq_lens: torch.Tensor, candidates: torch.Tensor, window: int,
                               n_valid: Optional[torch.Tensor], max_context: int, out_tokens: torch.Tensor,
                               seq_status: Optional[torch.Tensor] = None, out_logits: Optional[torch.Tensor] = None,
                               dump_seq_ids: Optional[torch.Tensor] = None, stream=None) -> None:
    """llm42_verify_window in the library's built-in scratch area (no workspace argument)."""
    num_seqs = seq_lens.numel()
    if candidates.shape != (num_seqs, window) or out_tokens.shape != (num_seqs, window):
        raise ValueError("candidates / out_tokens must be [num_seqs, window]")
    n_dump = 0 if dump_seq_ids is None else dump_seq_ids.numel()
    if n_dump and (out_logits is None or out_logits.shape[0] != n_dump or out_logits.shape[1] != window):
        raise ValueError("out_logits must be [n_dump, window, vocab]")
    kv = _kv_view(model, kv_base, num_blocks, block_table, num_seqs)
    _check(load_library().llm42_verify_window_static(
        model, ctypes.byref(kv), _ptr(seq_lens, torch.int32), _ptr(candidates, torch.int32), window,
        _ptr(n_valid, torch.int32), num_seqs, max_context, _ptr(out_tokens, torch.int32),
        _ptr(seq_status, torch.int32), _ptr(out_logits, torch.float32), _ptr(dump_seq_ids, torch.int32), n_dump,
        _stream_handle(stream)))


def llm42_decode_step(model: int, kv_base: torch.Tensor, num_blocks: int, block_table: torch.Tensor,
                      seq_lens: torch.Tensor, tokens: torch.Tensor, max_context: int, out_tokens: torch.Tensor,
                      workspace: torch.Tensor, seq_status: Optional[torch.Tensor] = None, stream=None,
                      sampling: Optional[Sampling] = None) -> None:
    """sampling given: llm42_decode_step_sampled."""
    num_seqs = seq_lens.numel()
    if tokens.numel() != num_seqs or out_tokens.numel() != num_seqs:
        raise ValueError("tokens / out_tokens must hold one entry per sequence")
    kv = _kv_view(model, kv_base, num_blocks, block_table, num_seqs)
    args = (model, ctypes.byref(kv), _ptr(seq_lens, torch.int32), _ptr(tokens, torch.int32), num_seqs, max_context,
            _ptr(out_tokens, torch.int32), _ptr(seq_status, torch.int32), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if sampling is None:
        _check(load_library().llm42_decode_step(*args))
    else:
        _check(load_library().llm42_decode_step_sampled(*args, ctypes.byref(sampling)))


def llm42_prefill_workspace_bytes(model: int, max_seqs: int, chunk: int, max_context: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().llm42_prefill_workspace_bytes(model, max_seqs, chunk, max_context, ctypes.byref(out)))
    return out.value


def llm42_prefill(model: int, kv_base: torch.Tensor, num_blocks: int, block_table: torch.Tensor,
                  seq_lens: torch.Tensor, prompt_tokens: torch.Tensor, prompt_offsets: torch.Tensor,
                  max_prompt_len: int, chunk: int, max_context: int, out_next_tokens: torch.Tensor,
                  workspace: torch.Tensor, seq_status: Optional[torch.Tensor] = None, stream=None,
                  sampling: Optional[Sampling] = None) -> None:
    num_seqs = seq_lens.numel()
    if prompt_offsets.numel() != num_seqs + 1 or out_next_tokens.numel() != num_seqs:
        raise ValueError("prompt_offsets holds num_seqs + 1 entries, out_next_tokens one per sequence")
    kv = _kv_view(model, kv_base, num_blocks, block_table, num_seqs)
    _check(load_library().llm42_prefill(
        model, ctypes.byref(kv), _ptr(seq_lens, torch.int32), _ptr(prompt_tokens, torch.int32),
        _ptr(prompt_offsets, torch.int32), num_seqs, max_prompt_len, chunk, max_context,
        _ptr(out_next_tokens, torch.int32), _ptr(seq_status, torch.int32), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream_handle(stream),
        ctypes.byref(sampling) if sampling is not None else None))


def llm42_commit_rollback(candidates: torch.Tensor, out_tokens: torch.Tensor, n_valid: Optional[torch.Tensor],
                          seq_lens: torch.Tensor, committed_counts: torch.Tensor, committed_tokens: torch.Tensor,
                          rolled_back_counts: Optional[torch.Tensor] = None, stream=None) -> None:
    num_seqs, window = candidates.shape
    _check(load_library().llm42_commit_rollback(
        _ptr(candidates, torch.int32), _ptr(out_tokens, torch.int32), _ptr(n_valid, torch.int32), num_seqs, window,
        _ptr(seq_lens, torch.int32), _ptr(committed_counts, torch.int32), _ptr(committed_tokens, torch.int32),
        _ptr(rolled_back_counts, torch.int32), _stream_handle(stream)))


def llm42_schedule_info() -> str:
    return load_library().llm42_schedule_info().decode()


def llm42_measure_attention_plan(model: int, num_seqs: int, window: int, max_context: int) -> Dict:
    """How a call of this shape distributes its attention work (see llm42_measure.h)."""
    out = (ctypes.c_int64 * 5)()
    _check(load_library().llm42_measure_attention_plan(model, num_seqs, window, max_context, out))
    return {"item_keys": out[0], "direct": bool(out[1]), "may_take_sequences": bool(out[2]),
            "sequences_flag_offset": out[3], "streaming": bool(out[4])}


def llm42_profile_enable(kind, max_launches: int) -> None:
    """kind: a name from KERNEL_CLASSES, or None for every class."""
    k = -1 if kind is None else KERNEL_CLASSES.index(kind)
    _check(load_library().llm42_profile_enable(k, max_launches))


def llm42_profile_collect(capacity: int):
    """Returns [(class name, milliseconds)] in launch order and disables timing."""
    ms = (ctypes.c_float * capacity)()
    kinds = (ctypes.c_int32 * capacity)()
    n = ctypes.c_int32()
    _check(load_library().llm42_profile_collect(ms, kinds, capacity, ctypes.byref(n)))
    return [(KERNEL_CLASSES[kinds[i]], float(ms[i])) for i in range(n.value)]
