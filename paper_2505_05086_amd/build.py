"""Builds the HIP library in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libasi_hip.so")
SOURCES = ["asi_api.hip", "asi_kernels.hip", "asi_subspace.hip", "asi_long.hip", "asi_planes.hip", "asi_bf16.hip", "asi_gram.hip", "asi_orth.hip", "asi_ttm.hip", "asi_ttm_stream.hip", "asi_corr.hip", "asi_rank.hip"]
# packed-fp32 VALU forms are switched off for every HIP translation unit
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return res.returncode, res.stdout


def build(verbose: bool = False, jobs: int = 6) -> str:
    """Compile csrc/*.hip into libasi_hip.so (always recompiles; the translation units are
    compiled side by side).  Returns the library path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        results = list(pool.map(_run, cmds))
    log = "".join(out for _, out in results)
    if any(rc != 0 for rc, _ in results):
        raise RuntimeError("hipcc failed:\n" + log)
    rc, out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs)
    log += out
    if verbose:
        print(log)
    if rc != 0:
        raise RuntimeError("hipcc link failed:\n" + log)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
