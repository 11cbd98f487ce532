"""Build libpoly.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpoly.so")
SOURCES = ["api.hip", "gemm.hip", "attention.hip", "rowops.hip", "select.hip", "profile.hip", "rowlin.hip", "mlp.hip", "rowlayer.hip", "contexts.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 ops are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force: bool = True, verbose: bool = False) -> str:
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(HERE, "_build", os.path.splitext(src)[0] + ".o")
        objs.append(o)
        deps = [s, os.path.join(CSRC, "poly_dev.h"), os.path.join(CSRC, "rowtile.h"), os.path.join(HERE, "..", "include", "poly.h"), os.path.join(HERE, "..", "include", "poly_profile.h")]
        if not force and os.path.exists(o) and all(os.path.getmtime(o) >= os.path.getmtime(d) for d in deps):
            continue
        if src.endswith(".cpp"):   # host-only source
            cmd = ["hipcc", "-O3", "-std=c++17", "-fPIC", "-Wall", "-c", s, "-o", o]
        else:
            cmd = ["hipcc", *FLAGS, "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print(f"--- {src} failed:\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(f"--- {src}:\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
