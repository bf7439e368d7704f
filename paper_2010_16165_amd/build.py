"""Compile the HIP/C++ sources for gfx950: paper_2010_16165_amd/libfupr.so (the
product) and paper_2010_16165_amd/measure/libfupr_measure.so (the two measuring
kernels the benchmark prices its roofline figures beside)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfupr.so")
MEASURE_DIR = os.path.join(HERE, "measure")
MEASURE_LIB = os.path.join(MEASURE_DIR, "libfupr_measure.so")
SOURCES = ["host_passes.cpp", "tuning.cpp", "kernels.hip", "conv_tiled.hip", "conv_patch.hip",
           "stem_pool.hip", "conv1x1.hip", "conv1x1_pipe.hip", "resident.hip", "model.cpp",
           "static_workspace.hip"]
HEADERS = [os.path.join(ROOT, "include", "fupr.h")] + [
    os.path.join(CSRC, h) for h in ("layout.h", "device_utils.h", "conv16.h", "stem_pool.h",
                                    "tuning.h")]
MEASURE_SOURCES = [os.path.join(MEASURE_DIR, "peaks.hip")]
MEASURE_HEADERS = [os.path.join(ROOT, "include", "fupr_measure.h")]


def _stale(lib, deps):
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    return any(os.path.getmtime(d) > t for d in deps)


def is_stale():
    return (_stale(LIB, [os.path.join(CSRC, s) for s in SOURCES] + HEADERS)
            or _stale(MEASURE_LIB, MEASURE_SOURCES + MEASURE_HEADERS))


def _compile(sources, lib, verbose, jobs=8):
    """One hipcc per source (in parallel), then one link."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-inline-asm",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs, procs = [], []
    for src in sources:
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [hipcc] + flags + ["-x", "hip", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            for _, p in procs:
                if p.poll() is None:
                    p.wait()
                    break
    for cmd, p in procs:
        if p.wait() != 0:
            raise subprocess.CalledProcessError(p.returncode, cmd)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib]
    if verbose:
        print(" ".join(link))
    subprocess.run(link, check=True)


def build(force=True, verbose=False):
    if not force and not is_stale():
        return LIB
    _compile([os.path.join(CSRC, s) for s in SOURCES], LIB, verbose)
    _compile(MEASURE_SOURCES, MEASURE_LIB, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
