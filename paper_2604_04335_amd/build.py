"""Build the gfx950 shared library in-tree with hipcc (no JIT, no torch extension machinery)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libdit_attn.so")
SOURCES = ["api.cpp", "plan.cpp", "sched_dp.cpp", "attn_fwd.hip", "merge.hip", "sp_layout.hip", "noalloc.hip"]
# bench.py's measurement aid (matrix-pipe ceiling loops); a library of its own that the attention library never loads
PROBE_LIB_PATH = os.path.join(PKG_DIR, "libdit_probe.so")
PROBE_SOURCES = ["probe/mfma_ceiling.hip"]

# -packed-fp32-ops is switched off on purpose: the compiler must not form packed fp32 instructions.
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(sources, lib_path: str, verbose: bool, extra_flags=()) -> str:
    cmd = [hipcc_path(), *HIP_FLAGS, *extra_flags]
    for s in sources:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith((".hip", ".cpp")) else [path])
    tmp = lib_path + ".tmp"
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature; drop that noise.
    noise = ("packed-fp32-ops", "is not a recognized feature")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, lib_path)
    return lib_path


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile the attention library into libdit_attn.so next to this file; returns its path."""
    return _compile(SOURCES, LIB_PATH, verbose, extra_flags)


def build_probe(verbose: bool = False) -> str:
    """Compile bench.py's measurement aid into libdit_probe.so next to this file; returns its path."""
    return _compile(PROBE_SOURCES, PROBE_LIB_PATH, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe(verbose=True))
