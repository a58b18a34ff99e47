"""Builds libsfmp.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsfmp.so")
PROBE_LIB = os.path.join(HERE, "libsfmp_probe.so")  # the benchmark's streaming-read probe, not part of the product
SOURCES = ["sfmp_host.cpp", "sfmp_unpack.hip", "sfmp_decode.hip", "sfmp_prefill.hip", "sfmp_lut.hip", "sfmp_api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off for all device code of this library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-munsafe-fp-atomics", "-Wno-unused-command-line-argument",
         # the first scalar kernel arguments arrive in scalar registers (the GEMV kernels are written for it)
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


# Per-file flags.  The decode kernels' loops branch on scalar values (the width of an item, the end of a slab); left to
# its default the compiler rewrites these branches into its structured form for divergent control flow, some eight
# scalar instructions per item of a loop whose time is its instruction count.
FILE_FLAGS = {"sfmp_decode.hip": ["-mllvm", "-structurizecfg-skip-uniform-regions"]}


def _compile(src: str, objdir: str, extra) -> str:
    obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *FILE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    if src.endswith(".cpp"):
        cmd.insert(1, "-x")
        cmd.insert(2, "hip")
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    noise = ("packed-fp32-ops", "is not a recognized feature")
    for line in (r.stdout + r.stderr).splitlines():
        if line.strip() and not any(n in line for n in noise):
            sys.stderr.write(line + "\n")
    return obj


def build(verbose: bool = False, extra_flags=()) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, objdir, list(extra_flags)), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    if verbose:
        print("built", LIB)
    probe_obj = _compile("sfmp_probe.hip", objdir, list(extra_flags))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", probe_obj, "-o", PROBE_LIB],
                       capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link of the probe library failed")
    if verbose:
        print("built", PROBE_LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
