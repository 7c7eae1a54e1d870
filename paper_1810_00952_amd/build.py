"""Build librelayhip.so (HIP kernels for gfx950 + host planner) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librelayhip.so")
SOURCES = ["api.cpp", "graph.cpp", "plan.cpp", "igemm.hip", "igemm_fast.hip", "igemm_dma.hip", "igemm_lp.hip", "igemm_ws.hip", "lstm_step.hip", "stem_pool.hip", "conv3x3_c64.hip", "conv3x3_run.hip", "conv3x3s2.hip", "eltwise.hip", "static_ws.hip", "calibrate.hip", "stem_direct.hip", "conv_wgrad.hip"]
HEADERS = ["graph.h", "plan.h", "handles.h", "kernels.h", "device_utils.h", "igemm_epilogue.h", os.path.join("..", "..", "include", "relayhip.h")]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]
# Per-source additions.  igemm_ws.hip: its accumulators live across a loop that also holds the epilogue's
# VALU code; with the accumulators in AGPRs the compiler copies all of them to VGPRs and back on every
# trip, so keep MFMA results in VGPRs there (the kernel fits in 256).
EXTRA_FLAGS = {"igemm_ws.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        cmd = [_hipcc()] + FLAGS + EXTRA_FLAGS.get(src, []) + (["-x", "hip"] if src.endswith(".hip") else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {src} failed\n{out}\n")
        elif out.strip() and verbose:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    # every symbol must resolve: load the freshly linked file before it replaces the old one
    import ctypes
    ctypes.CDLL(tmp)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
