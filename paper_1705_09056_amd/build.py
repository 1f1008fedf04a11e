"""Builds the C-ABI library (HIP kernels for gfx950 + host API) in-tree with hipcc.

    python -m paper_1705_09056_amd.build [--force]

Objects go to ``_build/`` (git-ignored), the library to ``paper_1705_09056_amd/libdpsgd_hip.so``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libdpsgd_hip.so")

SOURCES = ["api.cpp", "mix.hip", "grad.hip", "grad_f32.hip", "grad_mlp_bf16.hip", "grad_resnet.hip", "conv_mfma.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _newer(target: str, deps) -> bool:
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = False, verbose: bool = True) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(ROOT, "include", "dpsgd.h"))
    jobs = []
    objs = []
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        obj = os.path.join(OBJDIR, src.replace(".", "_") + ".o")
        objs.append(obj)
        if force or not _newer(obj, [path] + headers):
            lang = ["-x", "hip"]
            jobs.append(["hipcc", *FLAGS, *lang, "-c", path, "-o", obj])

    def run(cmd):
        if verbose:
            print("[build]", os.path.basename(cmd[-3]), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        return cmd, r

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        for cmd, r in ex.map(run, jobs):
            err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), r.stderr))
            if verbose and err.strip():
                print(err)
    if force or jobs or not _newer(LIB, objs):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
