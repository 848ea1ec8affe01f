"""Builds libcsp.so (the HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcsp.so")
SOURCES = ["api.hip", "score.hip", "score_single.hip", "select.hip", "compact.hip", "decode.hip", "reprune.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]
# score_single.hip runs one wavefront per SIMD with every register in use: its MFMA results must
# land in the registers the vector ALU reads (the default, accumulation registers plus copies,
# doubles the footprint of the logits and spills)
# score_single.hip: MFMA results in ordinary vector registers (the kernel keeps its weights there
# between two stages), and no NaN handling around max/min (its inputs are finite or -inf; the one
# place that must recognise a NaN tests the bit pattern)
EXTRA = {"score_single.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans", "-Wno-inline-asm"]}


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature and says so once per file: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    if verbose and out.strip():
        print(out)


def build_lib(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmpdir = tempfile.mkdtemp(prefix="csp_build_")
    try:
        objs = [os.path.join(tmpdir, s + ".o") for s in SOURCES]
        cmds = [[hipcc] + FLAGS + EXTRA.get(s, []) + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        tmp = LIB + f".tmp{os.getpid()}"
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp], verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
