"""Builds libw4a8.so (gfx950 code object + host C ABI) with hipcc, in-tree.

    python -m paper_2311_05161_amd.build          # compile everything, link
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libw4a8.so")

# The quantizers must evaluate the definition one binary32 operation at a time (bit-exact
# contract with a CPU evaluation), so no mul+add contraction there.  The GEMM epilogue is free
# to use fused multiply-add.
SOURCES = {
    "api.hip": [],
    "act_quant.hip": ["-ffp-contract=off"],
    "weight_quant.hip": ["-ffp-contract=off"],
    "pack.hip": [],
    "gemm_decode.hip": [],
    "gemm_prefill.hip": [],
    "aqas_search.hip": ["-ffp-contract=off"],
    "ceilings.hip": [],
}

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math",
    # the compiler must not form packed-fp32 instructions on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    """Run hipcc; drop the host pass's harmless 'not a recognized feature' lines from stderr."""
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip():
        print(err, file=sys.stderr, flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def _compile(name: str, extra, verbose: bool) -> str:
    src = os.path.join(CSRC, name)
    obj = os.path.join(OBJ_DIR, name.replace(".hip", ".o"))
    cmd = [_hipcc(), *COMMON, *extra, "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    _run(cmd)
    return obj


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Always recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=7) as pool:
        objs = list(pool.map(lambda kv: _compile(kv[0], [*kv[1], *extra_flags], verbose),
                             SOURCES.items()))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    _run(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
