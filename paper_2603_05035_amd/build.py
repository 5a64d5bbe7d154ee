"""Builds the HIP shared library `libgelo.so` in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libgelo.so")
SOURCES = ["api.hip", "gemm_bf16.hip", "gemm_f32.hip", "sampler.hip", "factor.hip", "lu.hip", "structured.hip", "small.hip", "gemm_fp8.hip", "calibrate.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = False) -> str:
    """Compiles every source (always, also when a library is already there) and links libgelo.so."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, proc in procs:
        out, _ = proc.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)   # host pass does not know the GPU feature
        if proc.returncode != 0 or (verbose and out.strip()):
            sys.stderr.write(f"--- {src}\n{out}\n")
        failed |= proc.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH], check=True)
    return LIB_PATH


def build_sanitized(verbose: bool = False) -> str:
    """Host-side sanitizer target: api.hip's HOST code (argument checks, context and mixing-object life cycle)
    compiled with AddressSanitizer + UndefinedBehaviorSanitizer, linked with the other, uninstrumented objects of
    `build()` into libgelo_hostsan.so, plus the driver tests/host_sanitize/lifecycle.cpp -> lifecycle_hostsan (both beside libgelo.so).
    The GPU code is not instrumented.  Call build() first."""
    obj_dir = os.path.join(HERE, "_build")
    root = os.path.dirname(HERE)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    api_obj = os.path.join(obj_dir, "api_hostsan.o")
    lib = os.path.join(HERE, "libgelo_hostsan.so")           # beside libgelo.so, where the host-side tests look for it
    exe = os.path.join(HERE, "lifecycle_hostsan")
    cmds = [
        [HIPCC, *FLAGS, *san, "-c", os.path.join(CSRC, "api.hip"), "-o", api_obj],
        [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", api_obj,
         *[os.path.join(obj_dir, src.replace(".hip", ".o")) for src in SOURCES if src != "api.hip"], "-o", lib],
        [HIPCC, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-fno-omit-frame-pointer",
         "-I", os.path.join(root, "include"), "-I", "/opt/rocm/include", "-D__HIP_PLATFORM_AMD__",
         os.path.join(root, "tests", "host_sanitize", "lifecycle.cpp"), "-L", HERE, "-lgelo_hostsan", "-L", "/opt/rocm/lib", "-lamdhip64",
         "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib", "-o", exe],
    ]
    for cmd in cmds:
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
        if proc.returncode != 0 or (verbose and out.strip()):
            sys.stderr.write(out + "\n")
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed (host sanitizer target)")
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
    if "--sanitize" in sys.argv:
        print(build_sanitized(verbose=True))
