"""Build the verifier library (libllm42.so) for gfx950 with hipcc, in-tree.

`python -m paper_2601_17768_amd.build` compiles every .hip file under csrc/
into an object file (in parallel) and links them into
paper_2601_17768_amd/libllm42.so.  hipcc cross-compiles: no GPU is needed.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllm42.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # every fused multiply-add is written explicitly
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
    # the LDS-direct loads name M0 in their clobber lists (they do overwrite it); the compiler accepts that but
    # warns about every reserved register it sees there, once per inlined copy
    "-Wno-inline-asm",
]
# Per-file additions.  The attention kernels keep their MFMA accumulators in ordinary vector
# registers: the softmax rescales them with vector arithmetic at every step, and accumulators
# placed in the accumulation registers would be copied out and back each time.
FILE_FLAGS = {
    "attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
}


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def kernel_sources_digest() -> str:
    """sha256 over the kernel sources (csrc/*.hip and *.h, in name order): identifies the kernels a
    measurement was taken on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJ_DIR, os.path.basename(s)[:-4] + ".o") for s in srcs]

    def compile_one(pair):
        src, obj = pair
        cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(os.path.basename(src), []), "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        return src, r

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        for src, r in ex.map(compile_one, zip(srcs, objs)):
            noise = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                sys.stderr.write(r.stderr)
                raise RuntimeError(f"hipcc failed on {src}")
            if verbose and noise.strip():
                sys.stderr.write(noise + "\n")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stderr)
        raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build())
