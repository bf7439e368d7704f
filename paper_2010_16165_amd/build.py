"""Compile the HIP/C++ sources into paper_2010_16165_amd/libfupr.so for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfupr.so")
SOURCES = ["host_passes.cpp", "kernels.hip", "conv_tiled.hip", "conv_patch.hip", "stem_pool.hip", "conv1x1.hip", "conv1x1_pipe.hip", "resident.hip",
           "peaks.hip", "model.cpp"]
HEADERS = [os.path.join(ROOT, "include", "fupr.h"), os.path.join(CSRC, "layout.h"),
           os.path.join(CSRC, "device_utils.h"), os.path.join(CSRC, "conv16.h"), os.path.join(CSRC, "stem_pool.h")]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False):
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
