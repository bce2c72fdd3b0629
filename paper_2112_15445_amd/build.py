"""Build libsparseconv.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsparseconv.so")
SOURCES = ["slab.hip", "dense_mfma_f16.hip", "dense_mfma_i8.hip", "dense_mfma_pipe_f16.hip", "dense_mfma_pipe_i8.hip", "dense_mfma_nat_f16.hip", "dense_mfma_nat_i8.hip", "dense_mfma_pipe_nat_f16.hip", "dense_mfma_pipe_nat_i8.hip", "dense_mfma_dl_f16.hip", "dense_mfma_dl_i8.hip", "plan.hip", "gather.hip", "dense_mfma.hip", "dense_library.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, jobs: int = 8, incremental: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles, unless
    `incremental` (development: only sources newer than their object, or older than a header)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        if incremental and os.path.exists(obj):
            deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, h) for h in os.listdir(CSRC) if h.endswith((".h", ".inc"))]
            deps.append(os.path.join(ROOT, "include", "sparse_conv.h"))
            if all(os.path.getmtime(d) <= os.path.getmtime(obj) for d in deps):
                continue
        cmd = [hipcc, "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs + ["-ldl"])
    os.replace(tmp, LIB)
    return LIB


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        # the host pass does not know the device-only target feature; that warning is harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{text}")
        if text.strip():
            print(text, file=sys.stderr)


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
