"""Build libaxonn_linear.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2502_08145_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
# one translation unit per kernel family (the compile time is the kernels'), compiled side by side
UNITS = ["axonn_linear.hip", "kernels_k64.hip", "kernels_ring_large.hip", "kernels_ring_small.hip", "kernels_edge.hip"]
LIB_DIR = os.path.join(HERE, "lib")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(LIB_DIR, "libaxonn_linear.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # hipcc must not form packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    # direct_load16 names m0 as clobbered on purpose (it writes it); clang calls that register reserved
    "-Wno-inline-asm",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (looked at $HIPCC, PATH and /opt/rocm/bin)")


def source_id() -> str:
    """Short hash of the kernel sources (csrc/ and the C header) with comments and blank space taken out:
    names the code a measurement was taken with, so that a stored counter reading can be told from one
    of an older kernel, while a reworded comment does not orphan it."""
    import hashlib
    import re
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".hpp", ".h")))
    files.append(os.path.join(os.path.dirname(HERE), "include", "axonn_linear.h"))
    for f in files:
        text = open(f, "r", encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)          # block comments
        text = re.sub(r"//[^\n]*", "", text)                        # line comments (no string in these sources holds //)
        text = "\n".join(" ".join(l.split()) for l in text.splitlines() if l.strip())
        h.update(os.path.basename(f).encode())
        h.update(text.encode())
    return h.hexdigest()[:16]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False, extra=(), units=None, out: str = LIB) -> str:
    """Compile every translation unit (in parallel) and link them into the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(os.path.dirname(out), exist_ok=True)
    os.makedirs(OBJ_DIR, exist_ok=True)
    cc = hipcc()
    units = list(units or UNITS)
    objs = [os.path.join(OBJ_DIR, u.replace(".hip", ".o")) for u in units]
    cmds = [[cc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, u), "-o", o] for u, o in zip(units, objs)]
    with ThreadPoolExecutor(max_workers=min(len(cmds), os.cpu_count() or 1)) as ex:
        list(ex.map(lambda c: _run(c, verbose), cmds))
    _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out], verbose)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
