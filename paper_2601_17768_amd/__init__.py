"""MI355X-native verifier hot path of LLM-42 (decode-verify-rollback).

`paper_2601_17768_amd.binding` is the thin ctypes layer over the C-ABI library
built from csrc/; `paper_2601_17768_amd.workloads` makes seeded synthetic inputs.
Nothing is loaded at package import time.
"""
__all__ = ["binding", "workloads", "build"]
