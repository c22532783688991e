"""Builds libgrim_bcr.so (host packer + HIP kernels for gfx950) in-tree with hipcc.

Every source is compiled to an object of its own (in parallel), then linked; objects live under _build/.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgrim_bcr.so")
SOURCES = ["bcr_pack.cpp", "bcr_spmm_fma.hip", "bcr_spmm_mma.hip", "bcr_spmm_wide.hip", "bcr_spmm_gather.hip", "bcr_conv.hip", "bcr_conv_wide.hip", "bcr_spmv.hip", "bcr_rnn_seq.hip",
           "lstm_cell.hip"]
NOISE = "is not a recognized feature for this target"


def _flags():
    return ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-x", "hip",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", "-Wno-inline-asm",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l and l.strip())
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))
    if verbose and err:
        print(err)


def _stale(src: str, obj: str) -> bool:
    """An object is reused only while it is newer than its source and than every header (the sources share struct
    definitions: an object built against an older header would read a matrix at the wrong offsets)."""
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    deps = [src] + [os.path.join(d, f) for d in (CSRC, os.path.join(ROOT, "include")) for f in os.listdir(d)
                    if f.endswith((".h", ".hpp"))]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False, only=None) -> str:
    """Compile every source and link the library.  `only`: recompile the named sources plus whatever is out of date,
    reusing the other objects (a development shortcut; build() in __graft_entry__ compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    sources = list(SOURCES)
    objs = {s: os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in sources}
    todo = [s for s in sources if only is None or s in only or _stale(os.path.join(CSRC, s), objs[s])]
    jobs = min(len(todo), int(os.environ.get("MAX_JOBS", "8"))) or 1
    with ThreadPoolExecutor(jobs) as pool:
        list(pool.map(lambda s: _run([hipcc] + _flags() + ["-c", os.path.join(CSRC, s), "-o", objs[s]], verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [objs[s] for s in sources] + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, only=sys.argv[1:] or None))
