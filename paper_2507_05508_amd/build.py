"""Builds libmlmc.so (HIP, gfx950) in-tree with hipcc.  Run as `python -m paper_2507_05508_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libmlmc.so")
SOURCES = ["mlmc_api.hip", "mlmc_topk.hip", "mlmc_bits_agg.hip", "mlmc_vrtn.hip", "mlmc_stopk.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                   # every fp32/fp64 op is a single IEEE operation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (proc.stdout + proc.stderr).splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = False) -> str:
    """Compiles every source (in parallel, one hipcc per file) and links libmlmc.so; always recompiles."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    extra = os.environ.get("MLMC_EXTRA_HIPCC_FLAGS", "").split()   # development aid: extra -D switches for experiments
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"] + extra + ["-c", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc] + compile_flags + [os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=len(cmds)) as ex:
        outs = list(ex.map(_run, cmds))
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH]))
    if verbose and any(o.strip() for o in outs):
        print("\n".join(o for o in outs if o.strip()))
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
