"""ctypes binding of libfupr.so: the same calls as include/fupr.h, argument
marshalling only.  Host calls take and return numpy arrays; device calls take
DeviceTensor views of torch CUDA tensors (torch provides device memory and
streams, nothing else).  There is no CPU fallback: if the library is missing
the import fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# torch first: libfupr.so and torch must share ONE HIP runtime in the process, and
# the one torch ships is the one its allocator and streams belong to.  Loading
# libfupr.so before torch would bind it to another copy that sees no device.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfupr.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2010_16165_amd.build` "
        "(there is no fallback path)")
_lib = C.CDLL(LIB_PATH)

# ---- enums ------------------------------------------------------------------
FUPR_OK = 0
ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_MASK_EMPTY, ERR_BN_VAR = -1, -2, -3, -4, -5
ERR_WORKSPACE, ERR_ALIGN, ERR_LAUNCH, ERR_ARG, ERR_LIMIT, ERR_BN_SCALE = -6, -7, -8, -9, -10, -11
F32, BF16, F16 = 0, 1, 2
FUSE_BN, FUSE_RELU, FUSE_ADD, FUSE_SCATTER, FUSE_CAT = 1, 2, 4, 8, 16
CAT_ALIGN = 64   # FUPR_CAT_ALIGN
OP_CONV, OP_MAXPOOL, OP_AVGPOOL = 0, 1, 2
SHORTCUT_IDENTITY, SHORTCUT_SUBSAMPLE_PAD, SHORTCUT_PROJECTION = 0, 1, 2
SCHEDULE_AUTO, SCHEDULE_PER_LAYER = 0, 1
DTYPES = {"f32": F32, "bf16": BF16, "f16": F16}


class FuprError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {status_str(status)} ({status})")


# ---- structs ----------------------------------------------------------------
class ConvShape(C.Structure):
    _fields_ = [("K", C.c_int32), ("C", C.c_int32), ("R", C.c_int32), ("S", C.c_int32),
                ("stride", C.c_int32), ("pad", C.c_int32)]


class Tensor(C.Structure):
    _fields_ = [("N", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("C", C.c_int32),
                ("c_stride", C.c_int32), ("dt", C.c_int), ("ptr", C.c_void_p)]


class Residual(C.Structure):
    _fields_ = [("t", Tensor), ("spatial_stride", C.c_int32), ("c_offset", C.c_int32)]


class OpDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("in_", C.c_int32), ("res", C.c_int32), ("conv", ConvShape),
                ("packed", C.c_void_p), ("epilogue", C.c_uint32),
                ("res_spatial_stride", C.c_int32), ("res_c_offset", C.c_int32),
                ("keep_idx", C.c_void_p), ("in2", C.c_int32), ("in2_spatial_stride", C.c_int32)]


class GraphDesc(C.Structure):
    _fields_ = [("dt", C.c_int), ("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("n_ops", C.c_int32), ("ops", C.POINTER(OpDesc))]


class Bn(C.Structure):
    _fields_ = [("gamma", C.POINTER(C.c_float)), ("beta", C.POINTER(C.c_float)),
                ("mean", C.POINTER(C.c_float)), ("var", C.POINTER(C.c_float)), ("eps", C.c_float)]


class BnOut(C.Structure):
    _fields_ = [("gamma", C.POINTER(C.c_float)), ("beta", C.POINTER(C.c_float)),
                ("mean", C.POINTER(C.c_float)), ("var", C.POINTER(C.c_float))]


class OpStats(C.Structure):
    _fields_ = [("flops", C.c_double), ("bytes", C.c_double), ("M", C.c_int64),
                ("K", C.c_int32), ("C", C.c_int32), ("R", C.c_int32), ("S", C.c_int32),
                ("stride", C.c_int32), ("first_op", C.c_int32), ("n_ops", C.c_int32),
                ("kernel", C.c_char_p)]


_F = C.POINTER(C.c_float)
_U8 = C.POINTER(C.c_uint8)
_I32 = C.POINTER(C.c_int32)
_SH = C.POINTER(ConvShape)
_T = C.POINTER(Tensor)

# Every symbol include/fupr.h declares, with its C signature.
SIGNATURES = {
    "fupr_status_str": (C.c_char_p, [C.c_int32]),
    "fupr_fold": (C.c_int32, [_SH, _F, _F, _F, _F, _F, _F, C.c_float, C.c_uint32, _F, _F]),
    "fupr_xconv_fuse": (C.c_int32, [_SH, _F, C.POINTER(Bn), _SH, _F, C.POINTER(Bn), C.c_int32, _SH, _F,
                                    C.POINTER(Bn), _F, C.POINTER(BnOut), _F, _F]),
    "fupr_proj_concat": (C.c_int32, [_SH, _F, _F, _SH, _F, _F, _SH, _F, _F]),
    "fupr_prune_count": (C.c_int32, [C.c_int32, C.c_int32]),
    "fupr_select_filters": (C.c_int32, [_SH, _F, C.c_int32, C.c_int32, _U8]),
    "fupr_prune": (C.c_int32, [_SH, _F, _F, _U8, C.c_int32, _SH, C.POINTER(_F), _I32, _I32, _F, _F,
                               C.POINTER(_F)]),
    "fupr_packed_bytes": (C.c_size_t, [_SH, C.c_int]),
    "fupr_pack": (C.c_int32, [_SH, _F, _F, C.c_int, C.c_void_p]),
    "fupr_conv_fused": (C.c_int32, [_SH, _T, C.c_void_p, C.POINTER(Residual), C.c_uint32, _T,
                                    C.c_void_p]),
    "fupr_conv_cat_fused": (C.c_int32, [_SH, _T, _T, C.c_int32, C.c_void_p, C.POINTER(Residual),
                                        C.c_uint32, _T, C.c_void_p]),
    "fupr_conv_scatter_fused": (C.c_int32, [_SH, _T, C.c_void_p, C.c_void_p, C.c_uint32, _T,
                                            C.c_void_p]),
    "fupr_maxpool": (C.c_int32, [_T, C.c_int32, C.c_int32, C.c_int32, _T, C.c_void_p]),
    "fupr_global_avgpool": (C.c_int32, [_T, _T, C.c_void_p]),
    "fupr_conv_conv1x1_fused": (C.c_int32, [_SH, _T, C.c_void_p, C.POINTER(Residual), C.c_uint32, _T,
                                            _SH, C.c_void_p, C.c_uint32, _T, C.c_void_p]),
    "fupr_conv_maxpool_fused": (C.c_int32, [C.POINTER(ConvShape), _T, C.c_void_p, C.c_int32,
                                            C.c_int32, C.c_int32, _T, C.c_void_p]),
    "fupr_model_create": (C.c_int32, [C.POINTER(GraphDesc), C.POINTER(C.c_void_p)]),
    "fupr_model_destroy": (None, [C.c_void_p]),
    "fupr_model_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32]),
    "fupr_model_output_shape": (C.c_int32, [C.c_void_p, C.c_int32, _T]),
    "fupr_forward": (C.c_int32, [C.c_void_p, _T, _T, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fupr_static_workspace_bytes": (C.c_size_t, []),
    "fupr_forward_static": (C.c_int32, [C.c_void_p, _T, _T, C.c_void_p]),
    "fupr_forward_timed": (C.c_int32, [C.c_void_p, _T, _T, C.c_void_p, C.c_size_t, C.c_void_p, _F]),
    "fupr_model_op_stats": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(OpStats)]),
    "fupr_model_num_ops": (C.c_int32, [C.c_void_p]),
    "fupr_model_num_launches": (C.c_int32, [C.c_void_p]),
    "fupr_model_launch_stats": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(OpStats)]),
    "fupr_model_set_schedule": (C.c_int32, [C.c_void_p, C.c_int32]),
    "fupr_model_table_bytes": (C.c_size_t, [C.c_void_p]),
    "fupr_model_table_write": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "fupr_model_set_table": (C.c_int32, [C.c_void_p, C.c_void_p]),
    "fupr_model_set_side_streams": (C.c_int32, [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)]),
    "fupr_graph_create": (C.c_int32, [C.c_void_p, _T, _T, C.c_void_p, C.c_size_t, C.c_void_p,
                                      C.POINTER(C.c_void_p)]),
    "fupr_graph_launch": (C.c_int32, [C.c_void_p, C.c_void_p]),
    "fupr_graph_destroy": (None, [C.c_void_p]),
    "fupr_tuning_set": (C.c_int32, [C.c_char_p, C.c_char_p]),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def status_str(status):
    return _lib.fupr_status_str(int(status)).decode()


def _check(status, where):
    if status != FUPR_OK:
        raise FuprError(status, where)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a):
    return None if a is None else a.ctypes.data_as(_F)


def conv_shape(K, Cn, R, S, stride, pad):
    return ConvShape(int(K), int(Cn), int(R), int(S), int(stride), int(pad))


def shape_of(W, stride, pad):
    k, c, r, s = W.shape
    return conv_shape(k, c, r, s, stride, pad)


# ---- host calls ---------------------------------------------------------------

def fupr_fold(shape, W, conv_bias, gamma, beta, mean, var, eps, fuse_flags):
    W = _f32(W)
    vecs = [None if v is None else _f32(v) for v in (conv_bias, gamma, beta, mean, var)]
    W_out = np.empty_like(W)
    b_out = np.empty(shape.K, dtype=np.float32)
    st = _lib.fupr_fold(C.byref(shape), _fp(W), *[_fp(v) for v in vecs], C.c_float(eps),
                        int(fuse_flags), _fp(W_out), _fp(b_out))
    _check(st, "fupr_fold")
    return W_out, b_out


def _bn_struct(bn):
    """(struct, arrays kept alive) for a batch-norm dict of synth.resnets."""
    arrs = [_f32(bn[k]) for k in ("gamma", "beta", "mean", "var")]
    return Bn(*[_fp(a) for a in arrs], C.c_float(bn["eps"])), arrs


def fupr_xconv_fuse(conv1, bn1, conv2, bn2, shortcut, proj=None, bnp=None):
    """conv1, conv2, proj: conv dicts {"W", "stride", "pad"}; bn*: batch-norm dicts.
    Returns (conv1', bn1', conv2', bn2') in the same formats."""
    W1, W2 = _f32(conv1["W"]), _f32(conv2["W"])
    s1 = shape_of(W1, conv1["stride"], conv1["pad"])
    s2 = shape_of(W2, conv2["stride"], conv2["pad"])
    k1, c, r, s = W1.shape
    k2 = W2.shape[0]
    b1, keep1 = _bn_struct(bn1)
    b2, keep2 = _bn_struct(bn2)
    sp, Wp, bp, keep_p = None, None, None, None
    if proj is not None:
        Wp = _f32(proj["W"])
        sp = shape_of(Wp, proj["stride"], proj["pad"])
        bp, keep_p = _bn_struct(bnp)
    W1_out = np.empty((k1 + c, c, r, s), dtype=np.float32)
    W2_out = np.empty((k2, k1 + c, r, s), dtype=np.float32)
    outs = [np.empty(k1 + c, dtype=np.float32) for _ in range(4)]
    beta2 = np.empty(k2, dtype=np.float32)
    bo = BnOut(*[_fp(a) for a in outs])
    st = _lib.fupr_xconv_fuse(C.byref(s1), _fp(W1), C.byref(b1), C.byref(s2), _fp(W2), C.byref(b2),
                              int(shortcut), None if sp is None else C.byref(sp), _fp(Wp),
                              None if bp is None else C.byref(bp), _fp(W1_out), C.byref(bo),
                              _fp(W2_out), _fp(beta2))
    _check(st, "fupr_xconv_fuse")
    bn1f = {"gamma": outs[0], "beta": outs[1], "mean": outs[2], "var": outs[3], "eps": bn1["eps"]}
    bn2f = dict(bn2)
    bn2f["beta"] = beta2
    return ({"W": W1_out, "stride": conv1["stride"], "pad": conv1["pad"]}, bn1f,
            {"W": W2_out, "stride": conv2["stride"], "pad": conv2["pad"]}, bn2f)


def fupr_proj_concat(last, W, b, proj, Wp, bp):
    """Returns (shape, W_cat, b_cat) of the last convolution with the projection
    shortcut concatenated along the channels."""
    W, Wp = _f32(W), _f32(Wp)
    b = None if b is None else _f32(b)
    bp = None if bp is None else _f32(bp)
    c1p = (last.C + CAT_ALIGN - 1) // CAT_ALIGN * CAT_ALIGN
    W_out = np.empty((last.K, c1p + proj.C, 1, 1), dtype=np.float32)
    b_out = np.empty(last.K, dtype=np.float32)
    out = ConvShape()
    st = _lib.fupr_proj_concat(C.byref(last), _fp(W), _fp(b), C.byref(proj), _fp(Wp), _fp(bp),
                               C.byref(out), _fp(W_out), _fp(b_out))
    _check(st, "fupr_proj_concat")
    return out, W_out, b_out


def fupr_prune_count(n, permille):
    r = _lib.fupr_prune_count(int(n), int(permille))
    if r < 0:
        raise FuprError(r, "fupr_prune_count")
    return r


def fupr_select_filters(shape, W, norm, n_prune):
    W = _f32(W)
    mask = np.empty(shape.K, dtype=np.uint8)
    st = _lib.fupr_select_filters(C.byref(shape), _fp(W), int(norm), int(n_prune),
                                  mask.ctypes.data_as(_U8))
    _check(st, "fupr_select_filters")
    return mask


def fupr_prune(prod, Wp, bp, mask, cons, Wc):
    """Returns (keep_idx, Wp_out, bp_out, [Wc_out...])."""
    Wp = _f32(Wp)
    bp = None if bp is None else _f32(bp)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    Wc = [_f32(w) for w in Wc]
    n = len(cons)
    K_keep = C.c_int32(0)
    keep_idx = np.full(prod.K, -1, dtype=np.int32)
    Wp_out = np.zeros_like(Wp)
    bp_out = None if bp is None else np.zeros_like(bp)
    Wc_out = [np.zeros_like(w) for w in Wc]
    cons_arr = (ConvShape * max(n, 1))(*cons)
    wc_ptrs = (_F * max(n, 1))(*[_fp(w) for w in Wc])
    wo_ptrs = (_F * max(n, 1))(*[_fp(w) for w in Wc_out])
    st = _lib.fupr_prune(C.byref(prod), _fp(Wp), _fp(bp), mask.ctypes.data_as(_U8), n,
                         cons_arr, wc_ptrs, C.byref(K_keep), keep_idx.ctypes.data_as(_I32),
                         _fp(Wp_out), _fp(bp_out), wo_ptrs)
    _check(st, "fupr_prune")
    kk = K_keep.value
    crs = prod.C * prod.R * prod.S
    Wp_c = Wp_out.reshape(-1)[:kk * crs].reshape(kk, prod.C, prod.R, prod.S).copy()
    bp_c = None if bp_out is None else bp_out[:kk].copy()
    Wc_c = []
    for sh, w in zip(cons, Wc_out):
        Wc_c.append(w.reshape(-1)[:sh.K * kk * sh.R * sh.S].reshape(sh.K, kk, sh.R, sh.S).copy())
    return keep_idx[:kk].copy(), Wp_c, bp_c, Wc_c


def fupr_packed_bytes(shape, dt):
    return int(_lib.fupr_packed_bytes(C.byref(shape), int(dt)))


def fupr_pack(shape, W, bias, dt):
    W = _f32(W)
    bias = None if bias is None else _f32(bias)
    nbytes = fupr_packed_bytes(shape, dt)
    if nbytes == 0:
        raise FuprError(ERR_SHAPE, "fupr_packed_bytes")
    blob = np.empty(nbytes, dtype=np.uint8)
    st = _lib.fupr_pack(C.byref(shape), _fp(W), _fp(bias), int(dt), blob.ctypes.data_as(C.c_void_p))
    _check(st, "fupr_pack")
    return blob


# ---- device tensors -----------------------------------------------------------

def _torch():
    import torch
    return torch


def _torch_dtype(dt):
    torch = _torch()
    return {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}[dt]


def min_c_stride(c, dt):
    a = 4 if dt == F32 else 8
    return (c + a - 1) // a * a


class DeviceTensor:
    """An NHWC activation tensor in device memory: a torch tensor of shape
    (N, H, W, c_stride) whose lanes C..c_stride-1 are zero."""

    def __init__(self, data, channels, dt):
        self.data = data
        self.C = int(channels)
        self.dt = int(dt)

    @classmethod
    def empty(cls, n, h, w, c, dt, c_stride=None, device="cuda:0"):
        torch = _torch()
        cs = c_stride or min_c_stride(c, dt)
        return cls(torch.empty((n, h, w, cs), dtype=_torch_dtype(dt), device=device), c, dt)

    @classmethod
    def from_nchw(cls, x, dt, c_stride=None, device="cuda:0"):
        """Upload an NCHW float array: one rounding (nearest even) to dt, NHWC, zero lanes."""
        torch = _torch()
        x = np.asarray(x)
        n, c, h, w = x.shape
        cs = c_stride or min_c_stride(c, dt)
        t = torch.zeros((n, h, w, cs), dtype=_torch_dtype(dt), device=device)
        src = torch.from_numpy(np.ascontiguousarray(x)).to(device)
        t[..., :c] = src.permute(0, 2, 3, 1).to(_torch_dtype(dt))
        return cls(t, c, dt)

    def to_nchw(self):
        """Download as an NCHW float64 array (exact widening)."""
        t = self.data[..., :self.C].permute(0, 3, 1, 2).to(_torch().float64)
        return t.cpu().numpy()

    def padding_is_zero(self):
        return bool((self.data[..., self.C:] == 0).all().item())

    @property
    def struct(self):
        n, h, w, cs = self.data.shape
        assert self.data.is_contiguous()
        return Tensor(n, h, w, self.C, cs, self.dt, self.data.data_ptr())


def upload_blob(blob, device="cuda:0"):
    """A host blob in device memory (torch's allocator aligns to >= 256 bytes)."""
    torch = _torch()
    t = torch.from_numpy(blob).to(device)
    assert t.data_ptr() % 256 == 0
    return t


def current_stream():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


# ---- device calls -------------------------------------------------------------

def fupr_conv_fused(shape, x, packed, res, epilogue_flags, y, stream=None):
    """packed: torch uint8 CUDA tensor; res: None or (DeviceTensor, spatial_stride, c_offset)."""
    xs, ys = x.struct, y.struct
    r = None
    if res is not None:
        r = Residual(res[0].struct, int(res[1]), int(res[2]))
    st = _lib.fupr_conv_fused(C.byref(shape), C.byref(xs), C.c_void_p(packed.data_ptr()),
                              None if r is None else C.byref(r), int(epilogue_flags), C.byref(ys),
                              stream if stream is not None else current_stream())
    _check(st, "fupr_conv_fused")


def fupr_conv_cat_fused(shape, x1, x2, x2_stride, packed, res, epilogue_flags, y, stream=None):
    """The convolution over [x1 ; x2] (x2 read at spatial stride x2_stride); other
    arguments as in fupr_conv_fused."""
    x1s, x2s, ys = x1.struct, x2.struct, y.struct
    r = None
    if res is not None:
        r = Residual(res[0].struct, int(res[1]), int(res[2]))
    st = _lib.fupr_conv_cat_fused(C.byref(shape), C.byref(x1s), C.byref(x2s), int(x2_stride),
                                  C.c_void_p(packed.data_ptr()), None if r is None else C.byref(r),
                                  int(epilogue_flags), C.byref(ys),
                                  stream if stream is not None else current_stream())
    _check(st, "fupr_conv_cat_fused")


def fupr_conv_scatter_fused(shape, x, packed, keep_idx, epilogue_flags, y, stream=None):
    """packed: torch uint8 CUDA tensor; keep_idx: torch int32 CUDA tensor of shape.K entries;
    y is updated in place."""
    xs, ys = x.struct, y.struct
    st = _lib.fupr_conv_scatter_fused(C.byref(shape), C.byref(xs), C.c_void_p(packed.data_ptr()),
                                      C.c_void_p(keep_idx.data_ptr()), int(epilogue_flags),
                                      C.byref(ys), stream if stream is not None else current_stream())
    _check(st, "fupr_conv_scatter_fused")


def fupr_maxpool(x, k, stride, pad, y, stream=None):
    xs, ys = x.struct, y.struct
    st = _lib.fupr_maxpool(C.byref(xs), int(k), int(stride), int(pad), C.byref(ys),
                           stream if stream is not None else current_stream())
    _check(st, "fupr_maxpool")


def fupr_conv_conv1x1_fused(shape1, x, packed1, res, flags1, y, shape2, packed2, flags2, h, stream=None):
    """res: None or (DeviceTensor, spatial_stride, c_offset), as in fupr_conv_fused."""
    xs, ys, hs = x.struct, y.struct, h.struct
    r = None
    if res is not None:
        r = Residual(res[0].struct, int(res[1]), int(res[2]))
    st = _lib.fupr_conv_conv1x1_fused(C.byref(shape1), C.byref(xs), C.c_void_p(packed1.data_ptr()),
                                      None if r is None else C.byref(r), int(flags1), C.byref(ys),
                                      C.byref(shape2), C.c_void_p(packed2.data_ptr()), int(flags2),
                                      C.byref(hs), stream if stream is not None else current_stream())
    _check(st, "fupr_conv_conv1x1_fused")


def fupr_conv_maxpool_fused(shape, x, packed, pool_k, pool_stride, pool_pad, y, stream=None):
    xs, ys = x.struct, y.struct
    st = _lib.fupr_conv_maxpool_fused(C.byref(shape), C.byref(xs), C.c_void_p(packed.data_ptr()),
                                      int(pool_k), int(pool_stride), int(pool_pad), C.byref(ys),
                                      stream if stream is not None else current_stream())
    _check(st, "fupr_conv_maxpool_fused")


def fupr_global_avgpool(x, y, stream=None):
    xs, ys = x.struct, y.struct
    st = _lib.fupr_global_avgpool(C.byref(xs), C.byref(ys),
                                  stream if stream is not None else current_stream())
    _check(st, "fupr_global_avgpool")


def fupr_static_workspace_bytes():
    return int(_lib.fupr_static_workspace_bytes())


def fupr_tuning_set(name, value):
    """value: None (back to automatic), or anything str() turns into the switch's text."""
    v = None if value is None else str(value).encode()
    _check(_lib.fupr_tuning_set(name.encode(), v), "fupr_tuning_set")


# ---- model ----------------------------------------------------------------------

class Model:
    """Owns a fupr_model and the device blobs its operators point into."""

    def __init__(self, dt, in_shape, ops, keepalive, device="cuda:0", side_streams=3):
        self.dt = int(dt)
        self.in_shape = tuple(in_shape)
        self._keepalive = keepalive
        arr = (OpDesc * len(ops))(*ops)
        g = GraphDesc(self.dt, in_shape[0], in_shape[1], in_shape[2], len(ops), arr)
        h = C.c_void_p()
        st = _lib.fupr_model_create(C.byref(g), C.byref(h))
        _check(st, "fupr_model_create")
        self._h = h
        self._graphs = []
        # device buffers and streams are the caller's: the one-kernel schedule's table
        # is uploaded here, and the per-operator schedule is lent side streams
        nbytes = int(_lib.fupr_model_table_bytes(self._h))
        torch = _torch()
        if nbytes and torch.cuda.is_available():
            dev = torch.empty(nbytes, dtype=torch.uint8, device=device)
            assert dev.data_ptr() % 256 == 0
            host = np.empty(nbytes, dtype=np.uint8)
            _check(_lib.fupr_model_table_write(self._h, C.c_void_p(dev.data_ptr()),
                                               host.ctypes.data_as(C.c_void_p)),
                   "fupr_model_table_write")
            dev.copy_(torch.from_numpy(host))
            torch.cuda.synchronize()
            _check(_lib.fupr_model_set_table(self._h, C.c_void_p(dev.data_ptr())),
                   "fupr_model_set_table")
            self._keepalive = list(self._keepalive or []) + [dev]
        self._side = []
        if side_streams and torch.cuda.is_available():
            self.set_side_streams([torch.cuda.Stream(device=device) for _ in range(side_streams)])

    def __del__(self):
        try:
            for g in getattr(self, "_graphs", []):
                _lib.fupr_graph_destroy(g)
            if getattr(self, "_h", None):
                _lib.fupr_model_destroy(self._h)
        except Exception:
            pass

    @property
    def num_ops(self):
        return int(_lib.fupr_model_num_ops(self._h))

    def workspace_bytes(self, batch):
        return int(_lib.fupr_model_workspace_bytes(self._h, int(batch)))

    def output_shape(self, batch):
        t = Tensor()
        _check(_lib.fupr_model_output_shape(self._h, int(batch), C.byref(t)),
               "fupr_model_output_shape")
        return t

    @property
    def num_launches(self):
        return int(_lib.fupr_model_num_launches(self._h))

    def set_side_streams(self, streams):
        """torch.cuda.Stream objects the per-operator schedule may fork sub-batches onto."""
        arr = (C.c_void_p * max(len(streams), 1))(*[s.cuda_stream for s in streams])
        _check(_lib.fupr_model_set_side_streams(self._h, len(streams), arr),
               "fupr_model_set_side_streams")
        self._side = list(streams)

    def set_schedule(self, schedule):
        _check(_lib.fupr_model_set_schedule(self._h, int(schedule)), "fupr_model_set_schedule")

    @staticmethod
    def _stats(s):
        return {"flops": s.flops, "bytes": s.bytes, "M": s.M, "K": s.K, "C": s.C, "R": s.R,
                "S": s.S, "stride": s.stride, "first_op": s.first_op, "n_ops": s.n_ops,
                "kernel": s.kernel.decode()}

    def op_stats(self, batch, op):
        s = OpStats()
        _check(_lib.fupr_model_op_stats(self._h, int(batch), int(op), C.byref(s)),
               "fupr_model_op_stats")
        return self._stats(s)

    def launch_stats(self, batch, launch):
        s = OpStats()
        _check(_lib.fupr_model_launch_stats(self._h, int(batch), int(launch), C.byref(s)),
               "fupr_model_launch_stats")
        return self._stats(s)

    def alloc(self, batch, device="cuda:0"):
        """(output DeviceTensor, workspace torch tensor) for a batch size."""
        torch = _torch()
        t = self.output_shape(batch)
        out = DeviceTensor.empty(t.N, t.H, t.W, t.C, self.dt, t.c_stride, device)
        ws = torch.empty(self.workspace_bytes(batch), dtype=torch.uint8, device=device)
        assert ws.data_ptr() % 256 == 0
        return out, ws

    def fupr_forward(self, x, out, ws, stream=None):
        xs, ys = x.struct, out.struct
        st = _lib.fupr_forward(self._h, C.byref(xs), C.byref(ys), C.c_void_p(ws.data_ptr()),
                               ws.numel(), stream if stream is not None else current_stream())
        _check(st, "fupr_forward")

    def fupr_forward_static(self, x, out, stream=None):
        """The forward pass in the library's own fixed workspace (no allocation)."""
        xs, ys = x.struct, out.struct
        st = _lib.fupr_forward_static(self._h, C.byref(xs), C.byref(ys),
                                      stream if stream is not None else current_stream())
        _check(st, "fupr_forward_static")

    def fupr_forward_timed(self, x, out, ws, stream=None):
        xs, ys = x.struct, out.struct
        ms = np.zeros(self.num_ops, dtype=np.float32)
        st = _lib.fupr_forward_timed(self._h, C.byref(xs), C.byref(ys), C.c_void_p(ws.data_ptr()),
                                     ws.numel(),
                                     stream if stream is not None else current_stream(), _fp(ms))
        _check(st, "fupr_forward_timed")
        return ms

    def fupr_graph_create(self, x, out, ws, stream):
        xs, ys = x.struct, out.struct
        g = C.c_void_p()
        st = _lib.fupr_graph_create(self._h, C.byref(xs), C.byref(ys), C.c_void_p(ws.data_ptr()),
                                    ws.numel(), stream, C.byref(g))
        _check(st, "fupr_graph_create")
        self._graphs.append(g)
        return g

    @staticmethod
    def fupr_graph_launch(g, stream):
        _check(_lib.fupr_graph_launch(g, stream), "fupr_graph_launch")
