"""In-tree builds: the gfx950 HIP library (C-ABI) and the input-generator helper.

`build_all()` always recompiles; the `ensure_*` helpers compile only when the shared
object is missing, which is what tests, the smoke check and the bench use.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
REPO_DIR = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")

HIP_LIB = os.path.join(PKG_DIR, "libspd_hip.so")
INPUTS_LIB = os.path.join(PKG_DIR, "libspd_inputs.so")

HIP_SOURCES = ["spd_host.cpp", "spd_kernels_f32.hip", "spd_kernels_bf16.hip", "spd_forward.hip"]


def _run(cmd):
    print("[build]", " ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass of hipcc does not know the packed-fp32 feature flag and says so: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError(f"build step failed ({res.returncode}): {' '.join(cmd)}")


def _hipcc() -> str:
    for c in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def build_inputs() -> str:
    cc = shutil.which("gcc") or "gcc"
    _run([cc, "-O3", "-march=x86-64-v2", "-ffp-contract=off", "-fno-math-errno", "-fopenmp",
          "-shared", "-fPIC", os.path.join(PKG_DIR, "inputs_gen.c"), "-o", INPUTS_LIB])
    return INPUTS_LIB


def build_hip() -> str:
    objs = []
    common = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
              "-I", os.path.join(REPO_DIR, "include"), "-I", CSRC,
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wall", "-Wno-unused-function"]
    os.makedirs(os.path.join(PKG_DIR, "_build"), exist_ok=True)
    procs = []
    for src in HIP_SOURCES:
        obj = os.path.join(PKG_DIR, "_build", os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = [_hipcc(), *common, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        print("[build]", " ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip():
            print(out, flush=True)
        if p.returncode != 0:
            raise RuntimeError(f"build step failed ({p.returncode}): {' '.join(cmd)}")
    _run([_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", HIP_LIB, "-lpthread"])
    return HIP_LIB


def build_all() -> None:
    build_inputs()
    build_hip()


def ensure_inputs() -> str:
    if not os.path.exists(INPUTS_LIB):
        build_inputs()
    return INPUTS_LIB


def ensure_hip() -> str:
    if not os.path.exists(HIP_LIB):
        build_hip()
    return HIP_LIB


if __name__ == "__main__":
    build_all()
    print("built", HIP_LIB, INPUTS_LIB, file=sys.stderr)
