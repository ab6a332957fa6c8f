"""Builds libpme.so in-tree with hipcc for gfx950 (python paper_2503_17513_amd/csrc/build.py)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
ROOT = os.path.dirname(PKG)
OBJ = os.path.join(ROOT, "_build")
SOURCES = ["pme_api.hip", "rotate_generic.hip", "rotate_mfma.hip", "gemm_generic.hip", "gemm_mfma.hip", "gemm_decode.hip", "gemm_mxfp4.hip", "probes.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
LIB = os.path.join(PKG, "libpme.so")


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(verbose: bool = True, extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(i):
        return _run([hipcc, *FLAGS, *extra_flags, "-c", os.path.join(HERE, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as ex:
        outs = list(ex.map(one, range(len(SOURCES))))
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]))
    if verbose:
        for o in outs:
            if o.strip():
                print(o)
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(extra_flags=tuple(sys.argv[1:]))
