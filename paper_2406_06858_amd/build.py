"""Builds libflux_mi355.so (gfx950) in-tree with hipcc.  Usage: python -m paper_2406_06858_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libflux_mi355.so")
N_CFGS = 10

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops", "is not a recognized feature")
    err = "\n".join(ln for ln in r.stderr.splitlines() if not any(n in ln for n in noise))
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + r.stdout + err)
    return err


def build(verbose: bool = False, jobs: int | None = None) -> str:
    os.makedirs(OBJ, exist_ok=True)
    units = [(os.path.join(CSRC, "flux_api.hip"), os.path.join(OBJ, "flux_api.o"), [])]
    for i in range(1, N_CFGS + 1):
        units.append((os.path.join(CSRC, "flux_gemm_inst.hip"), os.path.join(OBJ, f"flux_gemm_cfg{i}.o"),
                      [f"-DFLUX_CFG_ID={i}"]))
    jobs = jobs or min(8, os.cpu_count() or 1, len(units))

    def compile_one(u):
        src, obj, extra = u
        msg = _run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj])
        if verbose and msg.strip():
            print(msg, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, units))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
