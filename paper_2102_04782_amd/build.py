"""Build ``libdaq.so`` for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
OUT = os.path.join(HERE, "libdaq.so")
OBJ = os.path.join(HERE, "_build")

# -ffp-contract=off: the rounding of each fp32/fp64 expression in the quantizer is part of its contract.
# packed-fp32-ops off: packed fp32 VALU forms are avoided on the test machines.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-Wno-pass-failed"]
NOISE = "packed-fp32-ops"   # hipcc's host pass warns that it does not know the feature: harmless


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build(verbose: bool = False) -> str:
    """One object per translation unit, compiled side by side (no device symbol crosses a unit), then one link."""
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    objs = [os.path.join(OBJ, os.path.basename(s)[:-4] + ".o") for s in sources()]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        list(pool.map(lambda so: _run(["hipcc", *FLAGS, *inc, "-c", so[0], "-o", so[1]], verbose), zip(sources(), objs)))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT], verbose)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
