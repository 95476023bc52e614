"""Build libroco.so (gfx950) in-tree with hipcc.  `python -m paper_2402_06262_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libroco.so")
SOURCES = ["api.hip", "decode.hip", "prefill_simple.hip", "prefill_mfma.hip", "select_compact.hip", "block.hip", "profile.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-instruction accumulators live in ordinary vector registers: no copies to and from the
    # accumulation registers around every tile
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; the RoCo library cannot be built")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    out = (proc.stdout + proc.stderr).strip()
    # the host pass does not know the gfx target feature; that warning is harmless noise
    out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
    if verbose and out:
        print(out, flush=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{out}")


def build_library(verbose: bool = True) -> str:
    """Compile every HIP source (one hipcc process each, side by side) and link them into one shared library next to
    this file; returns its path.  Objects go to a temporary folder: nothing but the library is left in the tree."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = hipcc_path()
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="roco_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        cmds = [[hipcc, *compile_flags, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=min(len(cmds), os.cpu_count() or 1)) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
    print(LIB_PATH)
    sys.exit(0)
