"""Builds libslp.so (the C-ABI library) in-tree with hipcc for gfx950.

    python -m paper_2403_11204_amd.build

Each translation unit is compiled to an object under _build/ and linked into
paper_2403_11204_amd/libslp.so.  The generator file is compiled with
floating-point contraction off: its float32 transforms are defined operation by
operation so that a CPU gets the same bits.
"""

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libslp.so")
BUILD = os.path.join(ROOT, "_build")

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are kept out of every device code object
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wno-unused-command-line-argument",
]
UNITS = {
    "api.hip": [],
    "rng.hip": ["-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt"],
    "elementwise.hip": [],
    "gemm.hip": [],
    "probe.hip": [],
    "accuracy.hip": [],
}


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(unit, extra, verbose):
    obj = os.path.join(BUILD, unit.replace(".hip", ".o"))
    cmd = [hipcc()] + COMMON + extra + ["-c", os.path.join(CSRC, unit), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"      # host pass does not know the device feature
    log = "\n".join(l for l in r.stdout.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (unit, log))
    if log.strip() and verbose:
        print(log, flush=True)
    return obj


def build(verbose=True):
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda kv: _compile(kv[0], kv[1], verbose), UNITS.items()))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


def build_tools(verbose=True):
    """Development tools beside the library: the stand-alone matrix-product timer (csrc/gemm_bench.hip)."""
    os.makedirs(BUILD, exist_ok=True)
    out = os.path.join(BUILD, "gemm_bench")
    cmd = [hipcc()] + [a for a in COMMON if a != "-fPIC"] + [os.path.join(CSRC, "gemm_bench.hip"), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on gemm_bench.hip:\n%s" % r.stdout)
    return out


if __name__ == "__main__":
    build(verbose="-q" not in sys.argv)
    print("built", OUT)
    if "--tools" in sys.argv:
        print("built", build_tools(verbose="-q" not in sys.argv))
