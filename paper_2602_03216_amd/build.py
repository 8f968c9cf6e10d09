"""Builds libtsa.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libtsa.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "budget.hip", "drift.hip", "gather_scatter.hip", "probe.hip", "attend.hip", "attend_split.hip"]
# -packed-fp32-ops is switched off: the compiler must not form packed fp32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# per-file additions (attend: let the register allocator place MFMA results in VGPRs or AGPRs
# per instruction instead of forcing every accumulator into AGPRs)
_ATTEND_FLAGS = os.environ.get("TSA_ATTEND_FLAGS", "-mllvm -amdgpu-mfma-vgpr-form").split()
EXTRA = {"attend.hip": _ATTEND_FLAGS, "attend_split.hip": _ATTEND_FLAGS, "probe.hip": _ATTEND_FLAGS}
_NOISE = "packed-fp32-ops"


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libtsa cannot be built")


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in proc.stderr.splitlines() if _NOISE not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), err))
    return err


def build_library(verbose: bool = False) -> str:
    hipcc = hipcc_path()
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        return obj, _run([hipcc, *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        results = list(pool.map(compile_one, SOURCES))
    msgs = [m for _, m in results if m.strip()]
    msgs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for o, _ in results], "-o", LIB_PATH + ".tmp"]))
    if verbose:
        for m in msgs:
            if m.strip():
                print(m)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
