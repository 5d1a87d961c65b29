"""Builds libspecverify.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspecverify.so")
SOURCES = ["attention.hip", "attention_reuse.hip", "spec_verify.hip", "forward.hip", "sampler.hip", "gemm.hip",
           "elementwise.hip", "probe.hip", "decode.hip", "lookahead.hip"]
# packed-fp32 instructions are disabled for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Per-source additions.  The attention kernels: matrix instructions take their accumulators in ordinary vector
# registers; left to its default the compiler parks them in the accumulation registers and copies all
# 32 of them out and back around every block's products (the rare rescaling is vector arithmetic).
# The GEMM kernels keep the default: several of their variants measured slower with this option.
SOURCE_FLAGS = {"attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
                "attention_reuse.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
OBJ_DIR = os.path.join(HERE, "_build")


def _hipcc() -> str:
    for c in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found: cannot build libspecverify.so")


def sources_newer_than_lib() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + \
           [os.path.join(HERE, "..", "include", f) for f in os.listdir(os.path.join(HERE, "..", "include"))]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = False, verbose: bool = False) -> str:
    if not force and not sources_newer_than_lib():
        return LIB
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    noise = "packed-fp32-ops"

    def report(r):
        if verbose or r.returncode:
            print("\n".join(l for l in (r.stdout + r.stderr).splitlines() if noise not in l and l.strip()))

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + SOURCE_FLAGS.get(src, []) + ["-c", "-o", obj, os.path.join(CSRC, src)]
        return obj, subprocess.run(cmd, capture_output=True, text=True)

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:   # one hipcc process per source
        done = list(pool.map(compile_one, SOURCES))
    for _, r in done:
        report(r)
    if any(r.returncode for _, r in done):
        raise RuntimeError("hipcc failed building libspecverify.so")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for o, _ in done],
                       capture_output=True, text=True)
    report(r)
    if r.returncode:
        raise RuntimeError("hipcc failed linking libspecverify.so")
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
