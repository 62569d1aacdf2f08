"""Builds liblora_mi355.so (HIP, gfx950 only) next to this file."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblora_mi355.so")
SOURCES = ["lora_api.hip", "bucket.hip", "shrink.hip", "gemm.hip", "gemm_rows128.hip", "gemm_staged.hip", "reduce_expand.hip",
           "calibrate.hip", "placement.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 arithmetic stays off: plain v_fma_f32 / v_add_f32 only
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        print(err, file=sys.stderr)
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print("built", LIB)
    return LIB


# Host code with AddressSanitizer and UndefinedBehaviorSanitizer; the device side of a source is compiled as always.
SAN_FLAGS = [f for opt in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                           "-fno-omit-frame-pointer") for f in ("-Xarch_host", opt)]
# the sources that hold host logic (argument checks, slot table, launch planning, placement); the others are
# kernels with a launcher each and come from the ordinary build
SAN_SOURCES = ["lora_api.hip", "placement.cpp"]


def build_sanitized(out_dir: str, driver_src: str) -> str:
    """Builds, under out_dir, a copy of the library whose host logic is instrumented (a CPU test aid: run by
    the tests that need no GPU) and links `driver_src`, a C++ program that calls it, into an executable with the
    sanitizer runtimes.  Returns the executable's path."""
    os.makedirs(out_dir, exist_ok=True)
    os.makedirs(OBJ, exist_ok=True)
    plain = [s for s in SOURCES if s not in SAN_SOURCES]
    missing = [s for s in plain if not os.path.exists(os.path.join(OBJ, os.path.splitext(s)[0] + ".o"))]
    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(_compile, missing))

    def compile_san(src: str) -> str:
        obj = os.path.join(out_dir, os.path.splitext(os.path.basename(src))[0] + ".san.o")
        flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g", *SAN_FLAGS]
        res = subprocess.run([HIPCC, *flags, "-c", src, "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed for {src}:\n{res.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_san, [os.path.join(CSRC, s) for s in SAN_SOURCES] + [driver_src]))
    objs += [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in plain]
    exe = os.path.join(out_dir, "host_driver")
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link (sanitized) failed:\n" + res.stderr)
    return exe


if __name__ == "__main__":
    build()
