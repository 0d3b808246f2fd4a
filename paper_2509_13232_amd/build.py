"""Builds ``libspo_hip.so`` (gfx950 only) from ``csrc/`` with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libspo_hip.so")
SOURCES = ["tracker_adv.hip", "sampler.hip", "pg_logits.hip", "pg_fused.hip", "pg_api.hip", "timing.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         # packed fp32 instructions are kept out of the device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def source_digest() -> str:
    """Digest of the kernel sources (csrc/*.hip, *.hpp): names the kernels a profile was taken from."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(CSRC, "*.h*"))):
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


# host-side sanitizers (the device code cannot carry them): each -fsanitize= follows its own -Xarch_host
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _compile(src: str, obj_dir: str = OBJ, extra=()) -> str:
    obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on " + src)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    if verbose:
        print("built", LIB)
    return LIB


def build_sanitized_driver(driver_cpp: str, exe: str) -> str:
    """Links `driver_cpp` with the library's sources, host code built with AddressSanitizer and
    UndefinedBehaviorSanitizer, into the executable `exe` (a test aid: argument checks under sanitizers)."""
    obj_dir = OBJ + "_san"
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda src: _compile(src, obj_dir, SAN_FLAGS), SOURCES))
    drv_obj = os.path.join(obj_dir, "driver.o")
    steps = [
        ["g++", "-O1", "-g", "-std=c++17", "-I" + INCLUDE, "-fsanitize=address", "-fsanitize=undefined",
         "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-c", driver_cpp, "-o", drv_obj],
        # the sanitizer runtimes come from the host compiler that built the driver; hipcc adds the HIP runtime
        [_hipcc(), "--offload-arch=gfx950", drv_obj, *objs, "-o", exe, "-fsanitize=address", "-fsanitize=undefined"],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write((r.stdout + r.stderr)[-3000:])
            raise RuntimeError("sanitized build failed: " + " ".join(cmd[:2]))
    return exe


if __name__ == "__main__":
    build(verbose=True)
