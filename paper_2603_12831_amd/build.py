"""Build libomni_attn.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2603_12831_amd.build

Every source is compiled on each call; objects go to ``csrc/_build`` and the
library lands beside this file, where the binding looks for it.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libomni_attn.so")
SOURCES = ["api.hip", "decode_vector.hip", "decode_mfma.hip", "merge.hip", "debug.hip", "kv_cache.hip", "queues.hip"]
HOST_SOURCES = ["host_attn.cpp"]       # host-only C++ (no device code): compiled with the host compiler
HOST_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-pthread", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC]

# packed-fp32 instruction selection is switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # keep single-lane ticket atomics as issued (the wave-aggregation rewrite waits on them at once)
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build_library(verbose: bool = True, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(CSRC, "_build")
    os.makedirs(out, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(out, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if verbose and (r.stdout or r.stderr):
            keep = [ln for ln in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in ln]         # host pass does not know the device feature
            if keep:
                print("\n".join(keep), file=sys.stderr)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s" % src)
        return obj

    def compile_host(src):
        obj = os.path.join(out, src.replace(".cpp", ".o"))
        cxx = os.environ.get("CXX", "g++")
        r = subprocess.run([cxx, *HOST_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if verbose and (r.stdout or r.stderr):
            print(r.stdout + r.stderr, file=sys.stderr)
        if r.returncode != 0:
            raise RuntimeError("%s failed on %s" % (cxx, src))
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + len(HOST_SOURCES))) as ex:
        host_objs = [ex.submit(compile_host, s) for s in HOST_SOURCES]
        objs = list(ex.map(compile_one, SOURCES)) + [f.result() for f in host_objs]
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
