"""Build libzipccl.so (the codec) and libzipccl_yardstick.so (the benchmark's plain-copy kernel) in-tree with
hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libzipccl.so")
YARDSTICK = os.path.join(HERE, "libzipccl_yardstick.so")
SOURCES = ["zipccl_compress.hip", "zipccl_decompress.hip", "zipccl_aux.hip", "zipccl_host.cpp"]
HEADERS = [os.path.join(CSRC, "zipccl_internal.h"), os.path.join(CSRC, "zipccl_device.h"),
           os.path.join(ROOT, "include", "zipccl.h")]
TARGETS = {LIB: [os.path.join(CSRC, s) for s in SOURCES],
           YARDSTICK: [os.path.join(CSRC, "zipccl_yardstick.hip")]}


def stale(lib=LIB):
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    deps = TARGETS[lib] + HEADERS + [os.path.join(ROOT, "include", "zipccl_yardstick.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False, lib=None):
    """Compile every target (or the one named); returns the codec library's path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for target, sources in TARGETS.items():
        if (lib is not None and target != lib) or (not force and not stale(target)):
            continue
        tmp = target + f".{os.getpid()}.tmp"
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC]
        cmd += sources + ["-o", tmp]
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd)
        os.replace(tmp, target)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
