"""ctypes binding of libfupr_measure.so (include/fupr_measure.h): kernels of
known work for the benchmark's measured peaks.  Not part of the method."""
import ctypes as C
import os

import torch  # noqa: F401  (one HIP runtime per process: torch's)

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfupr_measure.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2010_16165_amd.build`")
_lib = C.CDLL(LIB_PATH)

SIGNATURES = {
    "fupr_measure_mfma": (C.c_int32, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.POINTER(C.c_double), C.c_void_p]),
    "fupr_measure_copy": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def fupr_measure_mfma(dt, shape, iters, workgroups, out):
    """out: torch float32 CUDA tensor of workgroups * 256 elements.  Returns the flops enqueued."""
    flops = C.c_double(0.0)
    st = _lib.fupr_measure_mfma(int(dt), int(shape), int(iters), int(workgroups),
                                C.c_void_p(out.data_ptr()), C.byref(flops), _stream())
    if st != 0:
        raise RuntimeError(f"fupr_measure_mfma: status {st}")
    return flops.value


def fupr_measure_copy(src, dst, nbytes):
    """src, dst: torch CUDA tensors of at least nbytes bytes."""
    st = _lib.fupr_measure_copy(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), int(nbytes),
                                _stream())
    if st != 0:
        raise RuntimeError(f"fupr_measure_copy: status {st}")
