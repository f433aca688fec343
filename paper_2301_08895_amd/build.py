"""Builds libabs.so (HIP kernels + host scheduler + C-ABI) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libabs.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIP_SOURCES = ["abs_api.hip", "kernels_regression.hip", "kernels_local.hip", "kernels_eval.hip", "kernels_mlp.hip",
               "calibrate.hip", "kernels_cnn.hip"]
CXX_SOURCES = ["sched.cpp"]

COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function"]
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    cc = hipcc()
    objs, procs = [], []
    for src in HIP_SOURCES + CXX_SOURCES:
        obj = os.path.join(OBJ_DIR, src.rsplit(".", 1)[0] + ".o")
        objs.append(obj)
        if src.endswith(".hip"):
            cmd = [cc, "-x", "hip"] + COMMON + HIP_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        else:
            cmd = ["g++"] + COMMON + ["-ffp-contract=off", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"compiling {src} failed:\n{out}")
        if verbose and out.strip():
            print(out)
    cmd = [cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"linking libabs.so failed:\n{r.stdout}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
