"""Builds libeh.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2407_21082_amd.build

The library is loaded by ``paper_2407_21082_amd.binding`` through ctypes; there
is no fallback path, so a missing or stale library is an error at import time
of the binding, not a silent slowdown.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libeh.so")
SOURCES = ["eh_api.hip", "eh_decode.hip", "eh_gemm.hip", "eh_gemm32.hip", "eh_calib.hip", "eh_probe.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function", *([f"-D{x}" for x in os.environ.get("EH_DEFINES", "").split()]),
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def build(verbose: bool = True) -> str:
    """Compiles every translation unit for gfx950 (in parallel) and links libeh.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = hipcc_path()
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc, *compile_flags, "-c", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
             os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    # The batched kernels wait for hand-counted loads; their device assembly is produced
    # alongside (same flags) and checked for register hazards before anything is linked.
    checked = [s for s in SOURCES if s.startswith("eh_gemm")]
    asms = [os.path.join(objdir, s.replace(".hip", ".s")) for s in checked]
    cmds += [[hipcc, *compile_flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"),
              "-I", CSRC, os.path.join(CSRC, s), "-o", a] for s, a in zip(checked, asms)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as ex:
        outs = list(ex.map(lambda c: _run(c, verbose), cmds))
    from . import check_gemm_asm
    for src, path in zip(checked, asms):
        with open(path) as f:
            findings, n_kernels, n_loads = check_gemm_asm.check_asm(f.read())
        if findings or n_kernels == 0:
            if os.path.exists(LIB):
                os.remove(LIB)
            raise RuntimeError(f"{src}: unsafe code generated for the hand-counted loads "
                               f"({n_kernels} kernels checked):\n" + "\n".join(findings[:10]))
        if verbose:
            print(f"check_gemm_asm {src}: {n_kernels} kernels, {n_loads} hand-counted loads, no hazard",
                  flush=True)
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", LIB], verbose))
    text = "\n".join(o for o in outs if o.strip())
    if verbose and text:
        print(text, flush=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
