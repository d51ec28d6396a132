"""Builds libtw.so (host packer + HIP kernels for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtw.so")
SOURCES = ["tw_pack.cpp", "tw_gemm.hip", "tw_dense.hip"]
HEADERS = ["tw_format.h", "tw_device.hpp", os.path.join("..", "..", "include", "tw.h")]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


# (source, -D flags, object): tw_gemm.hip is compiled as its host code (part 0) and eight groups of kernels
# (parts 1..4: fp16 / bf16 x plain / fused epilogue; 5..8: the same with the code for TEW blobs), all at once
UNITS = [("tw_pack.cpp", [], "tw_pack.cpp.o"), ("tw_dense.hip", [], "tw_dense.hip.o")] + [
    ("tw_gemm.hip", [f"-DTW_PART={i}"], f"tw_gemm.part{i}.o") for i in range(9)]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile for gfx950.  Packed-FP32 instruction selection is switched off for device code."""
    if not force and not needs_build():
        return LIB
    procs = []
    for src, defs, obj in UNITS:
        cmd = [hipcc(), "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"] + defs + [
               "-c", os.path.join(CSRC, src), "-o", os.path.join(CSRC, obj)]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, defs, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    failed = []
    for src, defs, pr in procs:
        _, stderr = pr.communicate()
        err = "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed.append(f"hipcc failed on {src} {' '.join(defs)}:\n{err}")
        elif verbose and err.strip():
            print(err, file=sys.stderr)
    if failed:
        raise RuntimeError("\n".join(failed))
    objs = [os.path.join(CSRC, obj) for _, _, obj in UNITS]
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
