"""Builds the HIP library (gfx950) in-tree: paper_2503_09716_amd/libmoe_mi355.so."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_mi355.so")
SOURCES = ["api.hip", "route.hip", "permute.hip", "ffn_gemm.hip", "combine.hip", "profile.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-Wno-unknown-attributes"]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, "common.h"), os.path.join(ROOT, "include", "moe.h")]
    jobs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        if force or _stale(o, [s] + headers):
            jobs.append(["hipcc", "-c", s, "-o", o] + FLAGS)

    def run(cmd):
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), err))
        if verbose and err.strip():
            print(err)

    with ThreadPoolExecutor(max_workers=5) as ex:
        list(ex.map(run, jobs))
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    if force or jobs or _stale(LIB, objs):
        run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    # a plain C program that calls the library through include/moe.h (run by the GPU tests)
    csrc = os.path.join(ROOT, "tests", "c_abi_check.c")
    cbin = os.path.join(HERE, "c_abi_check")
    if force or _stale(cbin, [csrc, LIB] + headers):
        run(["gcc", "-std=c99", "-O1", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROOT, "include"), "-I/opt/rocm/include",
             csrc, "-o", cbin, "-L" + HERE, "-lmoe_mi355", "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,$ORIGIN",
             "-Wl,-rpath,/opt/rocm/lib"])
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--force" in sys.argv, verbose=True))
