"""Builds, in-tree with hipcc for gfx950 only: libhsssvm.so (the product: C ABI of include/hss_svm.h),
libhsssvm_hooks.so (building-block entry points for the GPU unit tests, linked against the product library)
and native/hss_bench_native (a C driver of the ABI for hardware-counter runs)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhsssvm.so")
HOOKS_SRC = os.path.join(HERE, "csrc_test", "test_hooks.hip")
HOOKS_LIB = os.path.join(HERE, "libhsssvm_hooks.so")

FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result"]


ASAN_DIR = os.path.join(HERE, "_asan")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-omit-frame-pointer"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def build(verbose: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def one(src):
        obj = os.path.join(OBJ, src[:-4] + ".o")
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{res.stdout}\n{res.stderr}")
        if verbose and res.stderr.strip():
            print(res.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, sources()))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    # the unit tests' hooks: a library of their own that calls into the product library
    cmd = [hipcc, *FLAGS, "-shared", HOOKS_SRC, "-o", HOOKS_LIB, "-L" + HERE, "-lhsssvm", "-Wl,-rpath,$ORIGIN"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"test hooks failed:\n{res.stdout}\n{res.stderr}")
    # stand-alone driver of the C ABI (for hardware-counter runs that must wrap a plain executable)
    drv = os.path.join(HERE, "native", "hss_bench_native")
    cmd = [hipcc, "-O2", "-std=c++17", os.path.join(HERE, "native", "hss_bench_native.cpp"), "-o", drv,
           "-L" + HERE, "-lhsssvm", "-Wl,-rpath,$ORIGIN/.."]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"native driver failed:\n{res.stdout}\n{res.stderr}")
    build_sanitized(jobs)
    return LIB


def build_sanitized(jobs: int = 8) -> str:
    """The same library and native driver with AddressSanitizer + UndefinedBehaviorSanitizer on the HOST code only
    (device code is compiled as usual): _asan/libhsssvm.so and _asan/hss_bench_native.  tests/test_gpu_host_sanitizers.py
    runs the driver over the library's options and requires zero reports."""
    os.makedirs(ASAN_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["-O1", "-g"] + [f for f in FLAGS if f != "-O3"] + SAN_FLAGS

    def one(src):
        obj = os.path.join(ASAN_DIR, src[:-4] + ".o")
        res = subprocess.run([hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed on {src}:\n{res.stdout}\n{res.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, sources()))
    lib = os.path.join(ASAN_DIR, "libhsssvm.so")
    link = ["-fsanitize=address", "-fsanitize=undefined"]
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *link, "-o", lib, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link (sanitized) failed:\n{res.stdout}\n{res.stderr}")
    drv = os.path.join(ASAN_DIR, "hss_bench_native")
    res = subprocess.run([hipcc, "-O1", "-g", "-std=c++17", *link, os.path.join(HERE, "native", "hss_bench_native.cpp"),
                          "-o", drv, "-L" + ASAN_DIR, "-lhsssvm", "-Wl,-rpath,$ORIGIN"], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"native driver (sanitized) failed:\n{res.stdout}\n{res.stderr}")
    for o in objs:
        os.remove(o)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
