"""Builds libdash.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdash.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["dash.hip", "gemm.hip", "gemm_half.hip", "elementwise.hip", "power_iteration.hip", "model.hip"]

FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def build_library(verbose: bool = True) -> str:
    """Compiles every source (one hipcc process each, side by side) and links the shared library.
    Always compiles: nothing is taken from an earlier build."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(len(cmds), os.cpu_count() or 1)) as pool:
        outs = list(pool.map(lambda c: _run(c, verbose), cmds))
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose))
    if verbose:
        # the inline-assembly clobber notes of the direct-load helper repeat per instantiation: keep errors and
        # the rest readable
        text = "\n".join(o for o in outs if o)
        lines = [l for l in text.splitlines() if "clobber" not in l and "direct_load.h" not in l
                 and "s_mov_b32 m0" not in l and l.strip() not in ("^", "|")]
        if lines:
            print("\n".join(lines[-40:]))
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
