"""Builds the HIP library (gfx950) in-tree: paper_2504_15302_amd/libivf_mi355x.so.

Run as `python -m paper_2504_15302_amd.build` or through `__graft_entry__.build()`.
hipcc cross-compiles without a GPU.  The packed-fp32 feature is switched off for all
device code (the compiler would otherwise form packed fp32 instructions on its own).
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libivf_mi355x.so")
OBJ_DIR = os.path.join(HERE, "_build")

FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result"]


def _newer(target: str, sources) -> bool:
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(s) <= t for s in sources)


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "ivf.h"))
    objs = []
    for name in ("ivf_sort", "ivf_api", "ivf_worker"):
        src = os.path.join(CSRC, name + ".hip")
        obj = os.path.join(OBJ_DIR, name + ".o")
        deps = [src] + (headers if name != "ivf_sort" else [])
        # the sort unit only depends on its own source: skip it when unchanged
        if name == "ivf_sort" and _newer(obj, deps):
            objs.append(obj)
            continue
        if force or not _newer(obj, deps):
            cmd = ["hipcc", *FLAGS, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
        objs.append(obj)
    sched_src = os.path.join(CSRC, "ivf_sched.cpp")          # host-only arithmetic
    sched_obj = os.path.join(OBJ_DIR, "ivf_sched.o")
    cmd = ["hipcc", "-O2", "-fPIC", "-std=c++17", "-c", sched_src, "-o", sched_obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    objs.append(sched_obj)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    build_demo(verbose)
    return LIB


DEMO = os.path.join(HERE, "search_demo")


def build_demo(verbose: bool = False) -> str:
    """The plain-C consumer of the ABI (examples/search_demo.c), built with the host C
    compiler against the library and the system HIP runtime."""
    root = os.path.dirname(HERE)
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=gnu99", "-O1", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(root, "include"), os.path.join(root, "examples", "search_demo.c"),
           "-L" + HERE, "-livf_mi355x", "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", DEMO]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL if not verbose else None)
    return DEMO


if __name__ == "__main__":
    print(build(force="--force" in sys.argv or True, verbose=True))
