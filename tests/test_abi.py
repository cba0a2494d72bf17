"""The C-ABI library loads without a GPU, exports every function the header
declares, and rejects bad host-side arguments with the documented codes before
touching the device."""
import ctypes
import os
import re

import pytest

from helpers import ROOT
from paper_2601_17768_amd import binding as B

INCLUDE = os.path.join(ROOT, "include")


def declared_functions():
    """Every function any header under include/ declares."""
    names = set()
    for header in sorted(os.listdir(INCLUDE)):
        if header.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(INCLUDE, header)).read(), flags=re.S)
            names.update(re.findall(r"\b(llm42_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    assert "llm42_verify_window" in names and "llm42_commit_rollback" in names
    assert set(names) == set(B.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert b"v_mfma_f32_16x16x32_bf16" in lib.llm42_schedule_info()


def test_host_side_validation_needs_no_gpu():
    lib = B.load_library()
    out = ctypes.c_size_t()
    assert lib.llm42_workspace_bytes(None, 1, 8, 64, ctypes.byref(out)) == B.LLM42_EINVAL
    assert b"null" in lib.llm42_last_error()
    assert lib.llm42_kv_bytes(None, 4, ctypes.byref(out)) == B.LLM42_EINVAL
    assert lib.llm42_prefill_workspace_bytes(None, 1, 8, 64, None) == B.LLM42_EINVAL
    assert lib.llm42_commit_rollback(None, None, None, 1, 4, None, None, None, None, None) == B.LLM42_EINVAL
    assert lib.llm42_verify_window(None, None, None, None, 8, None, 1, 64, None, None, None, None, 0, None, 0,
                                   None) == B.LLM42_EINVAL
    handle = ctypes.c_void_p()
    w = B.Weights()
    good = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=688, vocab=1024,
                rope_theta=1e4, rms_eps=1e-5, kv_block_size=16, max_position=128)
    for bad, code in ((dict(head_dim=80), B.LLM42_ESHAPE), (dict(kv_block_size=32), B.LLM42_ESHAPE),
                      (dict(d_model=200), B.LLM42_ESHAPE), (dict(vocab=1000), B.LLM42_ESHAPE),
                      (dict(n_kv_heads=3), B.LLM42_ESHAPE), (dict(d_ffn=48), B.LLM42_ESHAPE), (dict(n_layers=0), B.LLM42_EINVAL),
                      (dict(rope_theta=0.0), B.LLM42_EINVAL)):
        cfg = B.Config(**{**good, **bad})
        assert lib.llm42_model_create(ctypes.byref(cfg), ctypes.byref(w), ctypes.byref(handle)) == code, bad
        assert handle.value is None
    # a good config with null weights is refused before any allocation
    cfg = B.Config(**good)
    assert lib.llm42_model_create(ctypes.byref(cfg), ctypes.byref(w), ctypes.byref(handle)) == B.LLM42_EINVAL


def test_kv_layout_round_trip():
    """The documented tile layout: K element ((f/8)*16 + t)*8 + f%8, V element f*16 + t."""
    import torch
    from paper_2601_17768_amd import kv_layout
    from paper_2601_17768_amd import workloads as wl
    shape = wl.TINY
    kv = kv_layout.alloc_kv(shape, 7, "cpu")
    ids = torch.tensor([5, 2, 6])
    n, hd = 37, shape.head_dim
    k = torch.randn(shape.n_layers, n, shape.n_kv_heads, hd).to(torch.bfloat16)
    v = torch.randn(shape.n_layers, n, shape.n_kv_heads, hd).to(torch.bfloat16)
    kv_layout.write_tokens(kv, ids, k[:, :20], v[:, :20], 0)
    kv_layout.write_tokens(kv, ids, k[:, 20:], v[:, 20:], 20)
    rk, rv = kv_layout.read_tokens(kv, ids, n, hd)
    assert torch.equal(rk, k) and torch.equal(rv, v)
    layer, pos, head, f = 1, 21, 1, 43
    tile_k = kv[layer, 0, ids[pos // 16], head]
    tile_v = kv[layer, 1, ids[pos // 16], head]
    t = pos % 16
    assert tile_k[((f // 8) * 16 + t) * 8 + f % 8] == k[layer, pos, head, f]
    assert tile_v[(((f // 16) * 4 + t // 4) * 16 + f % 16) * 4 + t % 4] == v[layer, pos, head, f]
    assert bool((kv[:, :, [0, 1, 3, 4]] == 0).all())        # other blocks untouched
