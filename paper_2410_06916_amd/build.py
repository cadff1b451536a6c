"""Builds libswift_hip.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libswift_hip.so")
SOURCES = ["swift_api.hip", "swift_kernels.hip", "swift_tiled.hip", "swift_opt.hip", "swift_sample.hip",
           "swift_attn_block.hip", "swift_attn_mfma.hip", "swift_gemm.hip"]
HEADERS = ["swift_kernels.h", "swift_device.h", "swift_attn.h", "swift_mv.h", os.path.join("..", "..", "include", "swift.h")]
# digest of the sources the library was built from, written beside it (file times do not survive every copy)
STAMP = os.path.join(HERE, "libswift_hip.srchash")
OBJ = os.path.join(HERE, "_build")

# packed-fp32 instruction selection is switched off for all device code
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-Wall", "-Wno-unused-result",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def lib_path() -> str:
    return LIB


def source_digest() -> str:
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for f in SOURCES + HEADERS:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(f.encode() + b"\0" + fh.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when there is no library, or it was built from other sources or flags than the present ones."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as fh:
        return fh.read().strip() != source_digest()


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compiles every source (one hipcc process per file, side by side) and links the library."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    cflags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as ex:
        jobs = [ex.submit(_run, [hipcc] + cflags + ["-c", os.path.join(CSRC, s), "-o", o], verbose)
                for s, o in zip(SOURCES, objs)]
        for j in jobs:
            j.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    with open(STAMP, "w") as fh:
        fh.write(source_digest() + "\n")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
