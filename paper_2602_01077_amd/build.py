"""Compiles the HIP sources under csrc/ into libpisa.so (in-tree, gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libpisa.so")
# (source, object name, extra flags).  The bf16 attention kernels are compiled with the compiler's
# iterative instruction scheduler, which gains them 2-5 % (measured; it does nothing for the other
# files and crashes the compiler on hetero.hip, so it is used for this one only).
ITERATIVE = ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp"]
UNITS = [("api.hip", "api", []), ("stats.hip", "stats", []), ("stats_bf16.hip", "stats_bf16", []),
         ("select.hip", "select", []), ("hetero.hip", "hetero", []), ("attn_fp32.hip", "attn_fp32", []),
         ("attn_bf16.hip", "attn_bf16", ITERATIVE),
         ("pairing.hip", "pairing", []), ("probe.hip", "probe", [])]
OBJ_DIR = os.path.join(PKG_DIR, "_build")


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = True) -> str:
    """Always recompiles; returns the path of the shared library."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    common = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wno-unused-command-line-argument", "-Wno-inline-asm",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objects = []
    procs = []
    for src, name, extra in UNITS:                       # the units compile side by side
        obj = os.path.join(OBJ_DIR, name + ".o")
        objects.append(obj)
        cmd = common + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    noise = "is not a recognized feature for this target"
    for cmd, pr in procs:
        _, stderr = pr.communicate()
        err = "\n".join(l for l in stderr.splitlines() if noise not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + err)
        if verbose and err.strip():
            print(err, file=sys.stderr)
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objects, verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
