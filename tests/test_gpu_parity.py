"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Tolerances: max-norm relative error max|gpu - ref| / max|ref| per tensor of at
most 2e-2 for bf16 / fp16 storage and 1e-3 for the fp32 path, and at least 99.9 %
of a tensor's elements within |gpu - ref| <= atol + rtol |ref| with rtol the same
tolerance and atol = rtol x the root mean square of the tensor's non-zero elements.  Masks and
kept-filter indices must be identical.
"""
import zlib

import numpy as np
import pytest

import synth
from oracle import reference as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-3, "bf16": 2e-2, "f16": 2e-2}


@pytest.fixture(scope="module")
def fx():
    import torch
    from paper_2010_16165_amd import binding as B, network
    assert torch.cuda.is_available()
    return B, network, torch


PASS_RATE = 0.999


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def pass_rate(got, ref, tol):
    """Share of elements with |got - ref| <= atol + rtol |ref|, rtol = tol and
    atol = tol x the root mean square of the tensor's NON-ZERO reference elements:
    the scale below which an element is the remainder of cancelled terms and a
    relative bound says nothing.  (Zeros are left out of the scale because a
    tensor behind a ReLU is mostly zeros: the sums that were clipped had the
    magnitude of those that survived, not of the tensor's mean square.)"""
    if not ref.size:
        return 1.0
    nz = ref[ref != 0]
    scale = float(np.sqrt(np.mean(np.square(nz)))) if nz.size else 0.0
    return float(np.mean(np.abs(got - ref) <= tol * scale + tol * np.abs(ref)))


def parity(got, ref, dtype, quiet=False):
    """Both readings of the error bound: max-norm relative error within the
    tolerance of the storage type, and at least PASS_RATE of the elements within
    atol + rtol |ref|.  Returns the max-norm relative error."""
    tol = TOL[dtype]
    err, rate = rel_err(got, ref), pass_rate(got, ref, tol)
    if not quiet:
        print(f"  max-norm rel err {err:.3e}, element-wise pass rate {rate:.5f}", flush=True)
    assert err <= tol, (err, tol)
    assert rate >= PASS_RATE, (rate, err)
    return err


def round_to(x, dtype, torch):
    """x rounded once to the storage dtype, as float64 (what the device holds)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    td = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    return t.to(td).to(torch.float64).numpy()


# ---- single convolution sites -------------------------------------------------

CONV_CASES = [
    # name, N, C, H, W, K, R, stride, pad, residual kind, relu
    ("3x3 C16 K12", 2, 16, 32, 32, 12, 3, 1, 1, None, True),
    ("3x3 C12 K16 +id", 2, 12, 32, 32, 16, 3, 1, 1, "identity", True),
    ("3x3 C10 K16 s2 +optA", 3, 10, 17, 15, 16, 3, 2, 1, "optionA", True),
    ("3x3 C39 K64 +id", 2, 39, 8, 8, 64, 3, 1, 1, "identity", True),
    ("3x3 C64 K45", 1, 64, 28, 28, 45, 3, 1, 1, None, True),
    ("3x3 C45 K64 ragged M", 1, 45, 13, 11, 64, 3, 1, 1, "identity", True),
    ("7x7 C3 K64 s2", 2, 3, 64, 64, 64, 7, 2, 3, None, True),
    ("1x1 C64 K32", 2, 64, 14, 14, 32, 1, 1, 0, None, True),
    ("1x1 C32 K256 +res norelu", 2, 32, 14, 14, 256, 1, 1, 0, "identity", False),
    ("1x1 C256 K512 s2 proj", 2, 256, 14, 14, 512, 1, 2, 0, None, False),
    ("3x3 C180 K256", 1, 180, 14, 14, 256, 3, 1, 1, None, True),
    ("3x3 C41 K39 irregular", 2, 41, 19, 23, 39, 3, 1, 1, None, True),
    ("3x3 C227 K193 s2", 1, 227, 15, 15, 193, 3, 2, 1, None, True),
    ("1x1 fc C64 K10", 5, 64, 1, 1, 10, 1, 1, 0, None, False),
    ("1x1 fc C512 K1000", 3, 512, 1, 1, 1000, 1, 1, 0, None, False),
    ("3x3 C1 K1", 1, 1, 5, 5, 1, 3, 1, 1, None, False),
    ("3x3 C8 K359 tiny image", 1, 8, 3, 3, 359, 3, 1, 1, None, True),
    # tiles that run across image boundaries, several filter groups, every shortcut kind
    ("3x3 C64 K128 7x7 x5 images +id", 5, 64, 7, 7, 128, 3, 1, 1, "identity", True),
    ("3x3 C96 K200 s2 14x12 +optA", 3, 96, 14, 12, 200, 3, 2, 1, "optionA", True),
    ("3x3 C40 K72 s2 odd width", 2, 40, 10, 13, 72, 3, 2, 1, None, False),
    ("3x3 C32 K32 56x56", 2, 32, 56, 56, 32, 3, 1, 1, None, True),
    ("3x3 C45 K64 56x56 +id", 1, 45, 56, 56, 64, 3, 1, 1, "identity", True),
    # 1 x 1: filters in LDS / pipelined, ragged channel and filter counts, shortcuts
    ("1x1 C200 K24", 3, 200, 9, 11, 24, 1, 1, 0, None, True),
    ("1x1 C512 K64 +id norelu", 2, 512, 10, 10, 64, 1, 1, 0, "identity", False),
    ("1x1 C520 K100 ragged", 3, 520, 7, 9, 100, 1, 1, 0, None, True),
    ("1x1 C1024 K128", 1, 1024, 14, 14, 128, 1, 1, 0, None, True),
    ("1x1 C136 K300 s2 +optA-shaped", 2, 136, 12, 12, 300, 1, 2, 0, None, False),
    ("1x1 fc C2048 K1000", 4, 2048, 1, 1, 1000, 1, 1, 0, None, False),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("case", CONV_CASES, ids=[c[0] for c in CONV_CASES])
def test_conv_site(fx, case, dtype):
    name, n, c, h, w, k, r, stride, pad, rkind, relu = case
    if dtype == "f32" and c * k * r * r > 200000:
        pytest.skip("fp32 path is exercised on the small shapes")
    conv_site(fx, case, dtype)


def conv_site(fx, case, dtype):
    """One convolution with merged batch norm, shortcut and ReLU through
    fupr_conv_fused against the oracle's conv, BN, add, ReLU."""
    B, network, torch = fx
    name, n, c, h, w, k, r, stride, pad, rkind, relu = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    print(f"case={name} dtype={dtype}", flush=True)
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = (rng.standard_normal((k, c, r, r)) * np.sqrt(2.0 / (c * r * r))).astype(np.float32)
    bn = {"gamma": rng.uniform(0.5, 1.5, k).astype(np.float32),
          "beta": (rng.standard_normal(k) * 0.1).astype(np.float32),
          "mean": (rng.standard_normal(k) * 0.1).astype(np.float32),
          "var": rng.uniform(0.5, 1.5, k).astype(np.float32), "eps": 1e-5}
    dt = B.DTYPES[dtype]
    p = (h + 2 * pad - r) // stride + 1
    q = (w + 2 * pad - r) // stride + 1

    xr = round_to(x, dtype, torch)
    ref = orc.batchnorm(orc.conv2d(xr, wt, stride, pad), bn)
    res_arg, res_ref = None, None
    if rkind == "identity":
        rs = rng.standard_normal((n, k, p, q)).astype(np.float32)
        res_ref = round_to(rs, dtype, torch)
        res_arg = (B.DeviceTensor.from_nchw(rs, dt), 1, 0)
    elif rkind == "optionA":
        rc = max(4, (k // 2) // 4 * 4)
        rs = rng.standard_normal((n, rc, 2 * p, 2 * q)).astype(np.float32)
        res_ref = orc.shortcut_subsample_pad(round_to(rs, dtype, torch), k, 2)
        res_arg = (B.DeviceTensor.from_nchw(rs, dt), 2, 0)
    if res_ref is not None:
        ref = orc.add(ref, res_ref)
    if relu:
        ref = orc.relu(ref)

    sh = B.shape_of(wt, stride, pad)
    Wf, bf = B.fupr_fold(sh, wt, None, bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"],
                         B.FUSE_BN)
    packed = B.upload_blob(B.fupr_pack(sh, Wf, bf, dt))
    xd = B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.empty(n, p, q, k, dt)
    yd.data.fill_(7.0)   # padding lanes must be overwritten with zeros
    flags = (B.FUSE_RELU if relu else 0) | (B.FUSE_ADD if res_arg else 0)
    B.fupr_conv_fused(sh, xd, packed, res_arg, flags, yd)
    torch.cuda.synchronize()
    got = yd.to_nchw()
    assert yd.padding_is_zero()
    return parity(got, ref, dtype)


def kernel_of(B, dtype, case):
    """Name of the kernel fupr_conv_fused launches for a case under the current tuning
    switches, from a one-operator model on the host (its parameter address is never read)."""
    name, n, c, h, w, k, r, stride, pad, rkind, relu = case
    op = B.OpDesc(B.OP_CONV, 0, -1, B.conv_shape(k, c, r, r, stride, pad), 0x1000, 0, 1, 0)
    return B.Model(B.DTYPES[dtype], (c, h, w), [op], None).op_stats(n, 0)["kernel"]


# Every instantiation of the per-layer kernel families, forced through the tuning
# switches onto shapes with ragged channel / filter counts, both strides, with and
# without a shortcut, several tiles per workgroup (bench.py at another batch size
# may pick any of them).
PATCH_TILES = ["p_256x64", "p_256x48", "p_256x32", "p_128x64", "p_128x32", "p_64x64", "p_224x64",
               "p_224x32", "p_448x64", "p_128x64w", "p_448x32", "p_448x48", "p_64x32",
               # the same kernel on the 32 x 32 x 16 MFMA
               "q_448x64", "q_256x64", "q_256x32", "q_128x64", "q_64x64", "q_128x64w", "q_512x32",
               "q_384x64"]
FORCED_3X3 = [
    ("forced 3x3 C45 K72 +id 28x28 x9", 9, 45, 28, 28, 72, 3, 1, 1, "identity", True),
    ("forced 3x3 C40 K100 s2 26x30 x4", 4, 40, 26, 30, 100, 3, 2, 1, None, True),
    ("forced 3x3 C136 K39 14x14 x20 norelu", 20, 136, 14, 14, 39, 3, 1, 1, None, False),
]


@pytest.mark.parametrize("tile", range(len(PATCH_TILES)), ids=PATCH_TILES)
def test_every_3x3_tile_forced(fx, tile):
    B, network, torch = fx
    B.fupr_tuning_set("patch_tile", tile)
    try:
        ran = 0
        for case in FORCED_3X3:
            for dtype in ("bf16", "f16"):
                kernel = kernel_of(B, dtype, case)
                if kernel != "conv3x3" + PATCH_TILES[tile]:
                    print(f"  {case[0]}: tile does not fit ({kernel} runs)", flush=True)
                    continue
                conv_site(fx, case, dtype)
                ran += 1
        assert ran >= 2, "the forced tile ran on too few shapes"
    finally:
        B.fupr_tuning_set("patch_tile", None)


PIPE_TILES = ["conv1x1p_128x128", "conv1x1p_128x64", "conv1x1p_64x64", "conv1x1q_128x128",
              "conv1x1q_128x256", "conv1x1q_256x128"]
STREAM_TILES = ["256f", "256f_c128", "128f", "64f", "64f_c512", "32f"]
FORCED_1X1 = [
    ("forced 1x1 C520 K100 +id 14x14 x11", 11, 520, 14, 14, 100, 1, 1, 0, "identity", True),
    ("forced 1x1 C136 K300 s2 24x20 x5", 5, 136, 24, 20, 300, 1, 2, 0, None, False),
    ("forced 1x1 C1024 K72 7x7 x30", 30, 1024, 7, 7, 72, 1, 1, 0, None, True),
    ("forced 1x1 C45 K256 +id 20x20 x6 norelu", 6, 45, 20, 20, 256, 1, 1, 0, "identity", False),
    ("forced 1x1 C64 K41 28x28 x5", 5, 64, 28, 28, 41, 1, 1, 0, None, True),
    ("forced 1x1 C256 K90 s2 12x12 x7", 7, 256, 12, 12, 90, 1, 2, 0, None, True),
    ("forced 1x1 C260 K257 +id 9x9 x9", 9, 260, 9, 9, 257, 1, 1, 0, "identity", True),   # one filter past a group of 256
    ("forced 1x1 C2048 K40 1x1 x3", 3, 2048, 1, 1, 40, 1, 1, 0, None, False),            # three pixels in all
    ("forced 1x1 C264 K136 s2 15x13 x3 +optionA", 3, 264, 15, 13, 136, 1, 2, 0, "optionA", True),
]


@pytest.mark.parametrize("tile", range(len(PIPE_TILES)), ids=PIPE_TILES)
def test_every_pipelined_1x1_tile_forced(fx, tile):
    B, network, torch = fx
    B.fupr_tuning_set("pipe_tile", tile)
    B.fupr_tuning_set("conv1x1_stream", 0)
    try:
        ran = 0
        for case in FORCED_1X1:
            for dtype in ("bf16", "f16"):
                if kernel_of(B, dtype, case) != PIPE_TILES[tile]:
                    continue
                conv_site(fx, case, dtype)
                ran += 1
        assert ran >= 4, "the forced tile ran on too few shapes"
        # two input tensors (the second at stride 2, ragged channel counts) through the same tile
        for case in CAT_CASES[2:4]:
            test_conv_cat_site(fx, case, "f16" if tile % 2 else "bf16")
    finally:
        B.fupr_tuning_set("pipe_tile", None)
        B.fupr_tuning_set("conv1x1_stream", None)


@pytest.mark.parametrize("order", [0, 1])
def test_pipelined_1x1_tile_orders(fx, order):
    """Both ways of handing tiles to workgroups (a contiguous range each; consecutive tiles
    per XCD), on layers with one and with several groups of filters."""
    B, network, torch = fx
    B.fupr_tuning_set("pipe_order", order)
    B.fupr_tuning_set("conv1x1_stream", 0)
    try:
        for case in (FORCED_1X1[0], FORCED_1X1[1], FORCED_1X1[2]):
            assert kernel_of(B, "bf16", case).startswith("conv1x1")
            conv_site(fx, case, "bf16")
        test_conv_cat_site(fx, CAT_CASES[3], "f16")
    finally:
        B.fupr_tuning_set("pipe_order", None)
        B.fupr_tuning_set("conv1x1_stream", None)


@pytest.mark.parametrize("tile", range(6), ids=STREAM_TILES)
def test_every_streaming_1x1_tile_forced(fx, tile):
    B, network, torch = fx
    B.fupr_tuning_set("stream_tile", tile)
    B.fupr_tuning_set("conv1x1_pipe", 0)
    try:
        ran = 0
        for case in FORCED_1X1:
            for dtype in ("bf16", "f16"):
                if kernel_of(B, dtype, case) != "conv1x1s_" + STREAM_TILES[tile]:
                    continue
                conv_site(fx, case, dtype)
                ran += 1
        assert ran >= 2, "the forced tile ran on too few shapes"
    finally:
        B.fupr_tuning_set("stream_tile", None)
        B.fupr_tuning_set("conv1x1_pipe", None)


GENERAL_TILES = ["64x16", "128x16", "64x32", "128x32", "64x48", "128x48", "64x64", "128x64",
                 "64x96", "128x96", "64x128", "128x128"]
FORCED_GENERAL = [
    ("forced general 3x3 C40 K100 s2 26x30 x4", 4, 40, 26, 30, 100, 3, 2, 1, None, True),
    ("forced general 3x3 C6 K20 +id 17x13 x3", 3, 6, 17, 13, 20, 3, 1, 1, "identity", True),
    ("forced general 1x1 C72 K200 +id 9x11 x5 norelu", 5, 72, 9, 11, 200, 1, 1, 0, "identity", False),
    ("forced general 5x5 C12 K33 s2 21x21 x2", 2, 12, 21, 21, 33, 5, 2, 2, None, True),
]


@pytest.mark.parametrize("tile", GENERAL_TILES)
def test_every_general_tile_forced(fx, tile):
    B, network, torch = fx
    B.fupr_tuning_set("conv_tile", "conv16t_" + tile)
    for family in ("conv_patch", "conv1x1_stream", "conv1x1_pipe"):
        B.fupr_tuning_set(family, 0)
    try:
        for case in FORCED_GENERAL:
            for dtype in ("bf16", "f16"):
                assert kernel_of(B, dtype, case) == "conv16t_" + tile
                conv_site(fx, case, dtype)
    finally:
        for family in ("conv_tile", "conv_patch", "conv1x1_stream", "conv1x1_pipe"):
            B.fupr_tuning_set(family, None)


@pytest.mark.parametrize("tile", [4, 5, 12], ids=["128x32", "64x64", "64x32"])
def test_small_tiles_with_several_units_in_flight(fx, tile):
    """The small tiles of the 3 x 3 kernel load up to three units ahead through a ring
    of LDS buffers.  The planner picks them for small layers only (one tile per
    workgroup); forced onto layers with more tiles than compute units, every
    workgroup walks several tiles and the ring wraps across tile boundaries."""
    B, network, torch = fx
    cases = [(6, 45, 56, 56, 64, 1, "identity"), (5, 40, 30, 26, 72, 2, None), (7, 100, 28, 28, 33, 1, None)]
    B.fupr_tuning_set("patch_tile", tile)
    try:
        for n, c, h, w, k, stride, rkind in cases:
            rng = np.random.default_rng(1000 * tile + c)
            x = rng.standard_normal((n, c, h, w)).astype(np.float32)
            wt = (rng.standard_normal((k, c, 3, 3)) * np.sqrt(2.0 / (c * 9))).astype(np.float32)
            bias = (rng.standard_normal(k) * 0.1).astype(np.float32)
            p, q = (h + 2 - 3) // stride + 1, (w + 2 - 3) // stride + 1
            for dtype in ("bf16", "f16"):
                dt = B.DTYPES[dtype]
                ref = orc.conv2d(round_to(x, dtype, torch), round_to(wt, dtype, torch), stride, 1)
                ref = ref + bias.astype(np.float64)[None, :, None, None]
                res_arg = None
                if rkind:
                    rs = rng.standard_normal((n, k, p, q)).astype(np.float32)
                    ref = ref + round_to(rs, dtype, torch)
                    res_arg = (B.DeviceTensor.from_nchw(rs, dt), 1, 0)
                ref = orc.relu(ref)
                sh = B.shape_of(wt, stride, 1)
                packed = B.upload_blob(B.fupr_pack(sh, wt, bias, dt))
                xd = B.DeviceTensor.from_nchw(x, dt)
                yd = B.DeviceTensor.empty(n, p, q, k, dt)
                yd.data.fill_(3.0)
                B.fupr_conv_fused(sh, xd, packed, res_arg, B.FUSE_RELU | (B.FUSE_ADD if res_arg else 0), yd)
                torch.cuda.synchronize()
                err = parity(yd.to_nchw(), ref, dtype)
                print(f"tile {tile} C{c} K{k} s{stride} {dtype}: rel err {err:.3e}", flush=True)
                assert yd.padding_is_zero() and err <= TOL[dtype]
    finally:
        B.fupr_tuning_set("patch_tile", None)


def test_identity_weights_copy_input(fx):
    """x = xconv(x, W~) (Sec. IV-B-1): bit-exact on the device, every dtype."""
    B, network, torch = fx
    for dtype in ("bf16", "f16", "f32"):
        dt = B.DTYPES[dtype]
        c = 24
        rng = np.random.default_rng(5)
        x = rng.standard_normal((2, c, 9, 11)).astype(np.float32)
        wt = np.zeros((c, c, 3, 3), dtype=np.float32)
        wt[np.arange(c), np.arange(c), 1, 1] = 1.0
        sh = B.shape_of(wt, 1, 1)
        packed = B.upload_blob(B.fupr_pack(sh, wt, None, dt))
        xd = B.DeviceTensor.from_nchw(x, dt)
        yd = B.DeviceTensor.empty(2, 9, 11, c, dt)
        B.fupr_conv_fused(sh, xd, packed, None, 0, yd)
        torch.cuda.synchronize()
        assert np.array_equal(yd.to_nchw(), xd.to_nchw()), dtype


def test_in_place_identity_residual(fx):
    """y may be the identity shortcut's own buffer."""
    B, network, torch = fx
    dt = B.BF16
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 16, 8, 8)).astype(np.float32)
    rs = rng.standard_normal((2, 16, 8, 8)).astype(np.float32)
    wt = (rng.standard_normal((16, 16, 3, 3)) * 0.1).astype(np.float32)
    sh = B.shape_of(wt, 1, 1)
    packed = B.upload_blob(B.fupr_pack(sh, wt, None, dt))
    xd = B.DeviceTensor.from_nchw(x, dt)
    y1 = B.DeviceTensor.empty(2, 8, 8, 16, dt)
    r1 = B.DeviceTensor.from_nchw(rs, dt)
    B.fupr_conv_fused(sh, xd, packed, (r1, 1, 0), B.FUSE_ADD | B.FUSE_RELU, y1)
    r2 = B.DeviceTensor.from_nchw(rs, dt)
    B.fupr_conv_fused(sh, xd, packed, (r2, 1, 0), B.FUSE_ADD | B.FUSE_RELU, r2)
    torch.cuda.synchronize()
    assert np.array_equal(y1.to_nchw(), r2.to_nchw())


# ---- pools -----------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_maxpool_exact(fx, dtype):
    B, network, torch = fx
    dt = B.DTYPES[dtype]
    rng = np.random.default_rng(8)
    x = -np.abs(rng.standard_normal((3, 20, 15, 18))).astype(np.float32) - 0.5
    xd = B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.empty(3, 8, 9, 20, dt)
    yd.data.fill_(3.0)
    B.fupr_maxpool(xd, 3, 2, 1, yd)
    torch.cuda.synchronize()
    ref = orc.maxpool(round_to(x, dtype, torch), 3, 2, 1)
    assert np.array_equal(yd.to_nchw(), ref)
    assert yd.padding_is_zero()


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_global_avgpool(fx, dtype):
    B, network, torch = fx
    dt = B.DTYPES[dtype]
    rng = np.random.default_rng(9)
    x = rng.standard_normal((5, 44, 7, 7)).astype(np.float32) + 1.0
    xd = B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.empty(5, 1, 1, 44, dt)
    B.fupr_global_avgpool(xd, yd)
    torch.cuda.synchronize()
    ref = orc.global_mean(round_to(x, dtype, torch))[:, :, None, None]
    assert rel_err(yd.to_nchw(), ref) <= (1e-5 if dtype == "f32" else 5e-3)
    assert yd.padding_is_zero()


# ---- whole networks ----------------------------------------------------------------

# ---- stem convolution + max-pool in one kernel -------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("size", [(64, 64), (70, 58), (30, 26)], ids=["64x64", "70x58", "30x26"])
def test_stem_maxpool_fused(fx, size, dtype):
    """Table II's ImageNet stem as one operator: against the oracle's conv, BN,
    ReLU, max-pool, and bit for bit against the two separate kernels."""
    B, network, torch = fx
    h, w = size
    n, c, k = 3, 3, 64
    rng = np.random.default_rng(1000 + h)
    print(f"stem {h}x{w} {dtype}", flush=True)
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = (rng.standard_normal((k, c, 7, 7)) * np.sqrt(2.0 / (c * 49))).astype(np.float32)
    bn = {"gamma": rng.uniform(0.5, 1.5, k).astype(np.float32),
          "beta": (rng.standard_normal(k) * 0.1).astype(np.float32),
          "mean": (rng.standard_normal(k) * 0.1).astype(np.float32),
          "var": rng.uniform(0.5, 1.5, k).astype(np.float32), "eps": 1e-5}
    dt = B.DTYPES[dtype]
    sh_, sw_ = (h + 6 - 7) // 2 + 1, (w + 6 - 7) // 2 + 1
    p, q = (sh_ + 2 - 3) // 2 + 1, (sw_ + 2 - 3) // 2 + 1
    xr = round_to(x, dtype, torch)
    ref = orc.maxpool(orc.relu(orc.batchnorm(orc.conv2d(xr, wt, 2, 3), bn)), 3, 2, 1)

    sh = B.shape_of(wt, 2, 3)
    Wf, bf = B.fupr_fold(sh, wt, None, bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"],
                         B.FUSE_BN)
    packed = B.upload_blob(B.fupr_pack(sh, Wf, bf, dt))
    xd = B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.empty(n, p, q, k, dt)
    yd.data.fill_(7.0)
    B.fupr_conv_maxpool_fused(sh, xd, packed, 3, 2, 1, yd)
    torch.cuda.synchronize()
    got = yd.to_nchw()
    err = parity(got, ref, dtype)
    print(f"  max-norm rel err {err:.3e}", flush=True)
    assert err <= TOL[dtype], (size, dtype, err)
    # the two-kernel path: same accumulation order, one rounding each, max of rounded values
    mid = B.DeviceTensor.empty(n, sh_, sw_, k, dt)
    y2 = B.DeviceTensor.empty(n, p, q, k, dt)
    B.fupr_conv_fused(sh, xd, packed, None, B.FUSE_RELU, mid)
    B.fupr_maxpool(mid, 3, 2, 1, y2)
    torch.cuda.synchronize()
    err2 = rel_err(got, y2.to_nchw())
    print(f"  against conv + pool kernels {err2:.3e}", flush=True)
    assert err2 <= TOL[dtype] / 4


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", [(32, 256, 32, True), (64, 200, 64, True), (58, 256, 45, False),
                                  (45, 256, 90, True), (100, 240, 128, True), (64, 256, 70, False)],
                         ids=["32-256-32+res", "64-200-64+res", "58-256-45", "45-256-90+res",
                              "100-240-128+res", "64-256-70"])
def test_two_1x1_convolutions_in_one_kernel(fx, case, dtype):
    """A block's last 1 x 1 convolution and the next block's first one as one
    launch: both outputs against the oracle (the second from the first one's
    value rounded to the storage type), and against the two separate kernels."""
    B, network, torch = fx
    c, k1, k2, with_res = case
    n, hh, ww = 3, 9, 7
    rng = np.random.default_rng(500 + c + k2)
    print(f"pair {c}->{k1}->{k2} res={with_res} {dtype}", flush=True)
    dt = B.DTYPES[dtype]
    x = rng.standard_normal((n, c, hh, ww)).astype(np.float32)
    w1 = (rng.standard_normal((k1, c, 1, 1)) * np.sqrt(2.0 / c)).astype(np.float32)
    b1 = (rng.standard_normal(k1) * 0.1).astype(np.float32)
    w2 = (rng.standard_normal((k2, k1, 1, 1)) * np.sqrt(2.0 / k1)).astype(np.float32)
    b2 = (rng.standard_normal(k2) * 0.1).astype(np.float32)
    rs = rng.standard_normal((n, k1, hh, ww)).astype(np.float32)
    y_ref = orc.conv2d(round_to(x, dtype, torch), w1, 1, 0) + b1.astype(np.float64)[None, :, None, None]
    if with_res:
        y_ref = orc.add(y_ref, round_to(rs, dtype, torch))
    y_ref = orc.relu(y_ref)
    sh1, sh2 = B.shape_of(w1, 1, 0), B.shape_of(w2, 1, 0)
    p1 = B.upload_blob(B.fupr_pack(sh1, w1, b1, dt))
    p2 = B.upload_blob(B.fupr_pack(sh2, w2, b2, dt))
    xd = B.DeviceTensor.from_nchw(x, dt)
    rd = B.DeviceTensor.from_nchw(rs, dt)
    yd = B.DeviceTensor.empty(n, hh, ww, k1, dt)
    hd = B.DeviceTensor.empty(n, hh, ww, k2, dt)
    yd.data.fill_(7.0)
    hd.data.fill_(7.0)
    res = (rd, 1, 0) if with_res else None
    f1 = B.FUSE_RELU | (B.FUSE_ADD if with_res else 0)
    B.fupr_conv_conv1x1_fused(sh1, xd, p1, res, f1, yd, sh2, p2, B.FUSE_RELU, hd)
    torch.cuda.synchronize()
    y = yd.to_nchw()
    assert yd.padding_is_zero() and hd.padding_is_zero()
    err_y = parity(y, y_ref, dtype)
    # the second convolution reads what the device holds of y
    h_ref = orc.relu(orc.conv2d(y, w2, 1, 0) + b2.astype(np.float64)[None, :, None, None])
    err_h = parity(hd.to_nchw(), h_ref, dtype)
    print(f"  max-norm rel err y {err_y:.3e}, h {err_h:.3e}", flush=True)
    assert err_y <= TOL[dtype] and err_h <= TOL[dtype]
    # the two separate kernels
    y2 = B.DeviceTensor.empty(n, hh, ww, k1, dt)
    h2 = B.DeviceTensor.empty(n, hh, ww, k2, dt)
    B.fupr_conv_fused(sh1, xd, p1, res, f1, y2)
    B.fupr_conv_fused(sh2, y2, p2, None, B.FUSE_RELU, h2)
    torch.cuda.synchronize()
    assert torch.equal(yd.data, y2.data)
    assert rel_err(hd.to_nchw(), h2.to_nchw()) <= TOL[dtype] / 4


CAT_CASES = [
    # name, N, C1 (last conv's input), C2 (block input), K, P, Q, shortcut stride, then-second-conv K2 or 0
    ("cat 38+64 -> 256 s1 (streaming kernel)", 3, 38, 64, 256, 14, 14, 1, 0),
    ("cat 38+64 -> 256 s1 then 1x1 -> 30 (pair)", 3, 38, 64, 256, 12, 14, 1, 30),
    ("cat 64+256 -> 512 s2 (pipelined kernel)", 2, 64, 256, 512, 14, 14, 2, 0),
    ("cat 207+512 -> 300 s2 ragged", 2, 207, 512, 300, 7, 9, 2, 0),
    ("cat 12+40 -> 72 s2 odd extent", 3, 12, 40, 72, 9, 7, 2, 0),
    ("cat 96+24 -> 64 s1", 2, 96, 24, 64, 10, 10, 1, 0),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", CAT_CASES, ids=[c[0] for c in CAT_CASES])
def test_conv_cat_site(fx, case, dtype):
    """A projection shortcut accumulated in the accumulators of the block's last
    1 x 1 convolution (Sec. IV-B-1): the device runs ONE convolution over the two
    tensors, the oracle the original graph - two convolutions with their batch
    norms, the addition, the ReLU."""
    B, network, torch = fx
    name, n, c1, c2, k, p, q, stride, k2 = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    print(f"case={name} dtype={dtype}", flush=True)
    dt = B.DTYPES[dtype]

    def bn_of(kk):
        return {"gamma": rng.uniform(0.5, 1.5, kk).astype(np.float32),
                "beta": (rng.standard_normal(kk) * 0.1).astype(np.float32),
                "mean": (rng.standard_normal(kk) * 0.1).astype(np.float32),
                "var": rng.uniform(0.5, 1.5, kk).astype(np.float32), "eps": 1e-5}

    h = np.maximum(rng.standard_normal((n, c1, p, q)), 0).astype(np.float32)
    hx, wx = (p - 1) * stride + 1 + (stride - 1), (q - 1) * stride + 1 + (stride - 1)
    x = np.maximum(rng.standard_normal((n, c2, hx, wx)), 0).astype(np.float32)
    w3 = (rng.standard_normal((k, c1, 1, 1)) * np.sqrt(2.0 / c1)).astype(np.float32)
    wp = (rng.standard_normal((k, c2, 1, 1)) * np.sqrt(2.0 / c2)).astype(np.float32)
    bn3, bnp = bn_of(k), bn_of(k)
    ref = orc.relu(orc.add(orc.batchnorm(orc.conv2d(round_to(h, dtype, torch), w3, 1, 0), bn3),
                           orc.batchnorm(orc.conv2d(round_to(x, dtype, torch), wp, stride, 0), bnp)))
    sh3, shp = B.shape_of(w3, 1, 0), B.shape_of(wp, stride, 0)
    f3 = B.fupr_fold(sh3, w3, None, bn3["gamma"], bn3["beta"], bn3["mean"], bn3["var"], 1e-5, B.FUSE_BN)
    fp = B.fupr_fold(shp, wp, None, bnp["gamma"], bnp["beta"], bnp["mean"], bnp["var"], 1e-5, B.FUSE_BN)
    shc, wc, bc = B.fupr_proj_concat(sh3, f3[0], f3[1], shp, fp[0], fp[1])
    packed = B.upload_blob(B.fupr_pack(shc, wc, bc, dt))
    hd, xd = B.DeviceTensor.from_nchw(h, dt), B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.empty(n, p, q, k, dt)
    yd.data.fill_(7.0)
    if not k2:
        B.fupr_conv_cat_fused(shc, hd, xd, stride, packed, None, B.FUSE_RELU, yd)
        torch.cuda.synchronize()
        assert yd.padding_is_zero()
        parity(yd.to_nchw(), ref, dtype)
        return
    # followed by the next block's first convolution in the same launch: through the model
    w1 = (rng.standard_normal((k2, k, 1, 1)) * np.sqrt(2.0 / k)).astype(np.float32)
    b1 = (rng.standard_normal(k2) * 0.1).astype(np.float32)
    sh1 = B.shape_of(w1, 1, 0)
    p1 = B.upload_blob(B.fupr_pack(sh1, w1, b1, dt))
    # tensors: 0 = block input x; 1 = h (a stand-in 1 x 1 convolution of x at the stride); 2 = y; 3 = h'
    w0 = (rng.standard_normal((c1, c2, 1, 1)) * np.sqrt(2.0 / c2)).astype(np.float32)
    sh0 = B.shape_of(w0, stride, 0)
    p0 = B.upload_blob(B.fupr_pack(sh0, w0, None, dt))
    ops = [B.OpDesc(B.OP_CONV, 0, -1, sh0, p0.data_ptr(), B.FUSE_RELU, 1, 0),
           B.OpDesc(B.OP_CONV, 1, -1, shc, packed.data_ptr(), B.FUSE_RELU | B.FUSE_CAT, 1, 0, None, 0, stride),
           B.OpDesc(B.OP_CONV, 2, -1, sh1, p1.data_ptr(), B.FUSE_RELU, 1, 0)]
    m = B.Model(dt, (c2, hx, wx), ops, [p0, p1, packed])
    assert m.num_launches == 2 and m.launch_stats(n, 1)["kernel"] == "conv1x1s_256f+conv1x1"
    out, ws = m.alloc(n)
    m.fupr_forward(xd, out, ws)
    torch.cuda.synchronize()
    xr = round_to(x, dtype, torch)
    h_dev = round_to(orc.relu(orc.conv2d(xr, round_to(w0, dtype, torch), stride, 0)), dtype, torch)
    y_ref = orc.relu(orc.add(orc.batchnorm(orc.conv2d(h_dev, w3, 1, 0), bn3),
                             orc.batchnorm(orc.conv2d(xr, wp, stride, 0), bnp)))
    h2_ref = orc.relu(orc.conv2d(round_to(y_ref, dtype, torch), w1, 1, 0) + b1.astype(np.float64)[None, :, None, None])
    parity(out.to_nchw(), h2_ref, dtype)
    m.set_schedule(B.SCHEDULE_PER_LAYER)
    assert m.num_launches == 3
    out2, ws2 = m.alloc(n)
    m.fupr_forward(xd, out2, ws2)
    torch.cuda.synchronize()
    assert rel_err(out.to_nchw(), out2.to_nchw()) <= TOL[dtype] / 4


def test_conv_cat_rejects_bad_calls(fx):
    B, network, torch = fx
    dt = B.BF16
    w = np.zeros((16, B.CAT_ALIGN + 8, 1, 1), np.float32)
    sh = B.shape_of(w, 1, 0)
    packed = B.upload_blob(B.fupr_pack(sh, w, None, dt))
    h = B.DeviceTensor.empty(1, 4, 4, 20, dt)
    x = B.DeviceTensor.empty(1, 8, 8, 8, dt)
    y = B.DeviceTensor.empty(1, 4, 4, 16, dt)

    def expect(code, fn):
        with pytest.raises(B.FuprError) as e:
            fn()
        assert e.value.status == code

    B.fupr_conv_cat_fused(sh, h, x, 2, packed, None, 0, y)
    expect(B.ERR_ARG, lambda: B.fupr_conv_cat_fused(sh, h, x, 3, packed, None, 0, y))
    small = B.DeviceTensor.empty(1, 4, 4, 8, dt)
    expect(B.ERR_SHAPE, lambda: B.fupr_conv_cat_fused(sh, h, small, 2, packed, None, 0, y))
    wide = B.DeviceTensor.empty(1, 8, 8, 9, dt)
    expect(B.ERR_SHAPE, lambda: B.fupr_conv_cat_fused(sh, h, wide, 2, packed, None, 0, y))
    w3 = np.zeros((16, B.CAT_ALIGN + 8, 3, 3), np.float32)
    expect(B.ERR_SHAPE, lambda: B.fupr_conv_cat_fused(B.shape_of(w3, 1, 1), h, x, 2, packed, None, 0, y))
    h32, x32, y32 = (B.DeviceTensor.empty(1, 4, 4, 20, B.F32), B.DeviceTensor.empty(1, 8, 8, 8, B.F32),
                     B.DeviceTensor.empty(1, 4, 4, 16, B.F32))
    expect(B.ERR_DTYPE, lambda: B.fupr_conv_cat_fused(sh, h32, x32, 2, packed, None, 0, y32))
    torch.cuda.synchronize()


def test_config4_projection_blocks_at_full_batch(fx):
    """The four blocks of the largest workload whose projection shortcut runs inside
    their last convolution, each alone at the full batch of 256 images on seeded
    synthetic activations; the oracle (both raw convolutions, both literal batch
    norms, removed input channels as zeros, the addition, the ReLU) computes a sample
    of output pixels one by one."""
    B, network, torch = fx
    model, batch = synth.make_config(4)
    dtype = model["dtype"]
    dt = B.DTYPES[dtype]
    masks = orc.select_masks(model)
    plan = network.optimise(model)
    rng = np.random.default_rng(synth.BASE_SEED + 4005)
    cats = [L for L in plan["layers"] if L.cat_stride]
    assert len(cats) == 4
    for L in cats:
        bi = int(L.site[1:].split(".")[0])
        blk = model["blocks"][bi]
        conv3, bn3 = blk["convs"][2], blk["bns"][2]
        convp, bnp = blk["shortcut"]["conv"], blk["shortcut"]["bn"]
        stride = convp["stride"]
        keep2 = np.flatnonzero(masks[(bi, 1)])
        c1, c2, k = len(keep2), convp["W"].shape[1], conv3["W"].shape[0]
        stage = blk["stage"]
        p = 56 >> stage
        hx = p * stride
        h = np.maximum(rng.standard_normal((batch, c1, p, p), dtype=np.float32), 0.0)
        x = np.maximum(rng.standard_normal((batch, c2, hx, hx), dtype=np.float32), 0.0)
        print(f"{L.site}: [{c1} ; {c2} at stride {stride}] -> {k} on {batch}x{p}x{p}", flush=True)
        hd, xd = B.DeviceTensor.from_nchw(h, dt), B.DeviceTensor.from_nchw(x, dt)
        packed = B.upload_blob(B.fupr_pack(L.shape, L.W, L.bias, dt))
        yd = B.DeviceTensor.empty(batch, p, p, k, dt)
        B.fupr_conv_cat_fused(L.shape, hd, xd, stride, packed, None, B.FUSE_RELU, yd)
        torch.cuda.synchronize()
        pts = [(0, 0, 0), (0, p - 1, p - 1), (1, 0, 0), (batch // 2, 0, p - 1), (batch - 1, p - 1, 0),
               (batch - 1, p - 1, p - 1)]
        pts += [(int(rng.integers(batch)), int(rng.integers(p)), int(rng.integers(p))) for _ in range(40)]
        hc = np.zeros((len(pts), conv3["W"].shape[1], 1, 1))
        xc = np.zeros((len(pts), c2, 1, 1))
        for j, (n, pp, qq) in enumerate(pts):
            hc[j, keep2, 0, 0] = round_to(h[n, :, pp, qq], dtype, torch)
            xc[j, :, 0, 0] = round_to(x[n, :, pp * stride, qq * stride], dtype, torch)
        ref = orc.relu(orc.add(orc.batchnorm(orc.conv2d(hc, conv3["W"], 1, 0), bn3),
                               orc.batchnorm(orc.conv2d(xc, convp["W"], 1, 0), bnp)))[:, :, 0, 0]
        got = np.stack([yd.data[n, pp, qq, :k].double().cpu().numpy() for n, pp, qq in pts])
        parity(got, ref, dtype)
        del hd, xd, yd, packed, h, x


def test_two_1x1_convolutions_rejected_when_not_a_pair(fx):
    B, network, torch = fx
    w1 = np.zeros((512, 64, 1, 1), np.float32)   # 512 filters: two filter groups
    w2 = np.zeros((32, 512, 1, 1), np.float32)
    sh1, sh2 = B.shape_of(w1, 1, 0), B.shape_of(w2, 1, 0)
    p1 = B.upload_blob(B.fupr_pack(sh1, w1, np.zeros(512, np.float32), B.BF16))
    p2 = B.upload_blob(B.fupr_pack(sh2, w2, np.zeros(32, np.float32), B.BF16))
    xd = B.DeviceTensor.from_nchw(np.zeros((1, 64, 4, 4), np.float32), B.BF16)
    yd = B.DeviceTensor.empty(1, 4, 4, 512, B.BF16)
    hd = B.DeviceTensor.empty(1, 4, 4, 32, B.BF16)
    with pytest.raises(B.FuprError) as e:
        B.fupr_conv_conv1x1_fused(sh1, xd, p1, None, B.FUSE_RELU, yd, sh2, p2, B.FUSE_RELU, hd)
    assert e.value.status == B.ERR_LIMIT


def test_stem_maxpool_fused_rejects_other_shapes(fx):
    B, network, torch = fx
    wt = np.zeros((32, 3, 7, 7), np.float32)
    sh = B.shape_of(wt, 2, 3)
    packed = B.upload_blob(B.fupr_pack(sh, wt, np.zeros(32, np.float32), B.BF16))
    xd = B.DeviceTensor.from_nchw(np.zeros((1, 3, 32, 32), np.float32), B.BF16)
    yd = B.DeviceTensor.empty(1, 8, 8, 32, B.BF16)
    with pytest.raises(B.FuprError) as e:
        B.fupr_conv_maxpool_fused(sh, xd, packed, 3, 2, 1, yd)
    assert e.value.status == B.ERR_LIMIT


def test_imagenet_stem_and_pool_run_as_one_launch(fx):
    B, network, torch = fx
    model = synth.make_imagenet_basic_resnet(14, "bf16", (1, 1, 1, 1), 300, widths=(64, 8, 8, 12),
                                             size=64, classes=7)
    m, _ = network.build(network.optimise(model))
    assert m.num_launches == m.num_ops - 1
    assert m.launch_stats(2, 0)["kernel"] == "stem7x7_maxpool"
    x = synth.make_input(14, 2, model["in_shape"])
    xd = B.DeviceTensor.from_nchw(x, B.BF16)
    out, ws = m.alloc(2)
    m.fupr_forward(xd, out, ws)
    torch.cuda.synchronize()
    fused = out.data.clone()
    m.set_schedule(B.SCHEDULE_PER_LAYER)
    assert m.num_launches == m.num_ops
    m.fupr_forward(xd, out, ws)
    torch.cuda.synchronize()
    ref = out.data.float()
    assert float((fused.float() - ref).abs().max() / ref.abs().max()) <= TOL["bf16"] / 4


def run_network(B, network, torch, model, x, **options):
    plan = network.optimise(model, **options)
    m, sites = network.build(plan)
    dt = B.DTYPES[model["dtype"]]
    xd = B.DeviceTensor.from_nchw(x, dt)
    out, ws = m.alloc(x.shape[0])
    m.fupr_forward(xd, out, ws)
    torch.cuda.synchronize()
    y = out.to_nchw()
    if model["head"] is not None:
        y = y[:, :, 0, 0]
    return plan, m, y


def small_models():
    return [
        synth.make_block_model(11, "f32", 8, 10, 250),
        synth.make_cifar_resnet(12, "bf16", 2, 400, widths=(4, 8, 12), size=12),
        synth.make_imagenet_basic_resnet(13, "bf16", (1, 1, 1, 1), 300, widths=(4, 8, 8, 12), size=32,
                                         classes=7),
        synth.make_imagenet_bottleneck_resnet(14, "bf16", (2, 1, 1, 1), 500, widths=(4, 4, 8, 8),
                                              size=32, classes=5),
        synth.make_imagenet_bottleneck_resnet(15, "f16", (1, 2, 1, 1), permille_range=(100, 700),
                                              widths=(8, 8, 8, 12), size=32, classes=5),
    ]


@pytest.mark.parametrize("mi", range(5))
def test_small_network(fx, mi):
    B, network, torch = fx
    model = small_models()[mi]
    x = synth.make_input(77, 3, model["in_shape"])
    masks = orc.select_masks(model)
    ref = orc.forward(model, round_to(x, model["dtype"], torch), masks=masks)
    plan, m, y = run_network(B, network, torch, model, x)
    assert set(plan["masks"]) == set(masks)
    for key in masks:
        assert np.array_equal(plan["masks"][key], masks[key])
        assert np.array_equal(plan["keep_idx"][key], np.flatnonzero(masks[key]))
    err = parity(y, ref, model["dtype"])
    print(f"model {mi} {model['name']} end-to-end rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


def fusible_models():
    return [
        synth.make_cifar_resnet(21, "bf16", 2, 400, widths=(8, 16, 24), size=16, classes=5),
        synth.make_imagenet_basic_resnet(22, "f16", (1, 2, 1, 1), 300, widths=(8, 16, 16, 24), size=32,
                                         classes=7),
    ]


@pytest.mark.parametrize("mi", range(2))
def test_aggressively_fused_network(fx, mi):
    """Aggressive fusion (Sec. IV-B) through the same kernels: the dilated
    convolutions without an addition give the oracle's fused model, and (the
    rewrite being an equivalence) the oracle's original model; with the n - m
    prune-back of Alg. 1 they give the oracle's fused model with those filters
    zeroed."""
    B, network, torch = fx
    model = fusible_models()[mi]
    x = synth.make_input(78, 3, model["in_shape"])
    xr = round_to(x, model["dtype"], torch)
    fused = orc.aggressive_fuse(model)
    ref_fused = orc.forward(fused, xr)
    ref_original = orc.forward(model, xr)
    plan, m, y = run_network(B, network, torch, model, x, aggressive=True, prune_fused=False)
    assert not plan["masks"] and not any(L.add for L in plan["layers"])
    err = parity(y, ref_fused, model["dtype"])
    print(f"fused model {mi}: rel err {err:.3e} (vs original {rel_err(y, ref_original):.3e})", flush=True)
    assert err <= TOL[model["dtype"]]
    parity(y, ref_original, model["dtype"])
    masks = orc.select_masks(fused)
    ref_pruned = orc.forward(fused, xr, masks=masks)
    plan, m, y = run_network(B, network, torch, model, x, aggressive=True)
    assert set(plan["masks"]) == set(masks)
    for key in masks:
        assert np.array_equal(plan["masks"][key], masks[key])
    err = parity(y, ref_pruned, model["dtype"])
    print(f"fused + pruned-back model {mi}: rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


@pytest.mark.parametrize("name,stages", [("resnet20", 1), ("resnet20", 2), ("resnet18", 2)])
def test_fusion_option_x_of_n(fx, name, stages):
    """The paper's fusion option x/n (Sec. V, optimization setting; the axis of
    Tables V, VI, VIII): the first x stages aggressively fused and pruned back
    (n - m), the other stages pruned at p with their addition in the epilogue."""
    B, network, torch = fx
    model = synth.make_paper_workload(name)
    x = synth.make_input(84, 2, model["in_shape"])
    xr = round_to(x, model["dtype"], torch)
    part = orc.aggressive_fuse(model, stages=stages)
    masks = orc.select_masks(part)
    ref = orc.forward(part, xr, masks=masks)
    plan, m, y = run_network(B, network, torch, model, x, aggressive=True, fuse_stages=stages)
    assert set(plan["masks"]) == set(masks)
    for key in masks:
        assert np.array_equal(plan["masks"][key], masks[key])
    fused_blocks = sum(b["stage"] < stages for b in model["blocks"])
    assert sum(L.add for L in plan["layers"]) == len(model["blocks"]) - fused_blocks
    err = parity(y, ref, model["dtype"])
    print(f"{name} fused {stages} stages: rel err {err:.3e}", flush=True)


@pytest.mark.parametrize("name", synth.PAPER_WORKLOADS)
def test_paper_workload_at_batch_one(fx, name):
    """The networks the paper measures (Table II) in the setting it measures them
    in (one image, Tables V-VI), against the oracle."""
    B, network, torch = fx
    model = synth.make_paper_workload(name)
    x = synth.make_input(79, 1, model["in_shape"])
    masks = orc.select_masks(model)
    ref = orc.forward(model, round_to(x, model["dtype"], torch), masks=masks)
    plan, m, y = run_network(B, network, torch, model, x)
    # CIFAR networks: one kernel; ImageNet networks: one per operator, stem + pool as one
    assert m.num_launches == (1 if name in ("resnet20", "resnet32") else m.num_ops - 1)
    err = parity(y, ref, model["dtype"])
    print(f"{model['name']}: rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


def test_unpruned_cifar_network_stays_in_one_kernel(fx):
    """Unpruned ResNet-20: the 64 x 64 x 3 x 3 parameter blocks of the last stage do
    not fit LDS twice, so those layers stage their parameters at their own start;
    the network still runs as one kernel and matches the oracle."""
    B, network, torch = fx
    model = synth.make_paper_workload("resnet20", permille=0)
    x = synth.make_input(80, 3, model["in_shape"])
    ref = orc.forward(model, round_to(x, model["dtype"], torch))
    plan, m, y = run_network(B, network, torch, model, x)
    assert m.num_launches == 1
    err = parity(y, ref, model["dtype"])
    print(f"{model['name']}: rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


CONFIG_BATCH = {0: 1, 1: 8, 2: 2, 3: 2, 4: 2}


@pytest.mark.parametrize("idx", range(5))
def test_baseline_config_end_to_end(fx, idx):
    """The five workloads at their real layer shapes (reduced batch so the
    oracle finishes in seconds)."""
    B, network, torch = fx
    model, _ = synth.make_config(idx)
    n = CONFIG_BATCH[idx]
    x = synth.make_input(synth.BASE_SEED + idx, n, model["in_shape"])
    masks = orc.select_masks(model)
    print(f"config {idx}: oracle on {n} images", flush=True)
    ref = orc.forward(model, round_to(x, model["dtype"], torch), masks=masks)
    plan, m, y = run_network(B, network, torch, model, x)
    for key in masks:
        assert np.array_equal(plan["masks"][key], masks[key])
        assert np.array_equal(plan["keep_idx"][key], np.flatnonzero(masks[key]))
    assert np.isfinite(y).all()
    err = parity(y, ref, model["dtype"])
    print(f"config {idx} {model['name']} end-to-end rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_baseline_config_teacher_forced(fx, idx):
    """Every convolution site of the workload alone: the device site is fed
    the oracle's input (and shortcut) rounded to the storage type and must
    reproduce the oracle's output of that site."""
    B, network, torch = fx
    model, _ = synth.make_config(idx)
    dtype = model["dtype"]
    dt = B.DTYPES[dtype]
    x = synth.make_input(synth.BASE_SEED + idx, 1, model["in_shape"])
    masks = orc.select_masks(model)
    trace = []
    orc.forward(model, round_to(x, dtype, torch), masks=masks, trace=trace)
    by_site = {t["site"]: t for t in trace}
    plan = network.optimise(model, concat_projection=False)   # one operator per convolution site
    # which (block, conv) feeds / is each site, to drop removed channels
    worst = 0.0
    for L in plan["layers"]:
        t = by_site[L.site]
        xin, res, yref = t["x"], t["res"], t["y"]
        if L.site == "fc":
            xin = xin[:, :, None, None]
            yref = yref[:, :, None, None]
        if L.site.startswith("b") and ".conv" in L.site:
            bi = int(L.site[1:].split(".")[0])
            ci = int(L.site.split("conv")[1]) - 1
            if (bi, ci - 1) in masks:      # input produced by a pruned conv
                xin = xin[:, np.flatnonzero(masks[(bi, ci - 1)])]
            if (bi, ci) in masks:          # this conv lost filters
                yref = yref[:, np.flatnonzero(masks[(bi, ci)])]
        packed = B.upload_blob(B.fupr_pack(L.shape, L.W, L.bias, dt))
        xd = B.DeviceTensor.from_nchw(xin, dt)
        n, k, p, q = yref.shape
        yd = B.DeviceTensor.empty(n, p, q, k, dt)
        res_arg = None
        if res is not None:
            res_arg = (B.DeviceTensor.from_nchw(res, dt), 1, 0)
        flags = (B.FUSE_RELU if L.relu else 0) | (B.FUSE_ADD if res_arg else 0)
        B.fupr_conv_fused(L.shape, xd, packed, res_arg, flags, yd)
        torch.cuda.synchronize()
        err = parity(yd.to_nchw(), yref, dtype, quiet=True)
        worst = max(worst, err)
        assert err <= TOL[dtype], (L.site, err)
    print(f"config {idx}: worst site rel err {worst:.3e} over {len(plan['layers'])} sites", flush=True)


def resident_models():
    return [
        synth.make_cifar_resnet(31, "bf16", 3, 400),
        synth.make_cifar_resnet(32, "f16", 2, 250, widths=(8, 24, 40), size=24, classes=13),
        synth.make_block_model(33, "bf16", 16, 32, 250),
        synth.make_cifar_resnet(34, "bf16", 1, 250, widths=(16, 32, 64), size=32),
    ]


@pytest.mark.parametrize("mi", range(4))
def test_one_kernel_schedule_equals_per_layer_schedule(fx, mi):
    """The LDS-resident one-kernel schedule and the per-layer schedule compute
    the same network (the one-kernel schedule adds bias and shortcut inside the
    MFMA accumulation, so roundings differ): the two agree within half the
    tolerance, and both match the oracle."""
    B, network, torch = fx
    model = resident_models()[mi]
    n = 5
    x = synth.make_input(41 + mi, n, model["in_shape"])
    dt = B.DTYPES[model["dtype"]]
    plan = network.optimise(model)
    m, _ = network.build(plan)
    assert m.num_launches == 1, "model should be eligible for the one-kernel schedule"
    xd = B.DeviceTensor.from_nchw(x, dt)
    out_a, ws = m.alloc(n)
    out_a.data.fill_(9.0)
    m.fupr_forward(xd, out_a, ws)
    torch.cuda.synchronize()
    m.set_schedule(B.SCHEDULE_PER_LAYER)
    assert m.num_launches == m.num_ops
    out_b, ws_b = m.alloc(n)
    m.fupr_forward(xd, out_b, ws_b)
    torch.cuda.synchronize()
    between = rel_err(out_a.to_nchw(), out_b.to_nchw())
    assert between <= TOL[model["dtype"]] / 2, between
    assert out_a.padding_is_zero()
    masks = orc.select_masks(model)
    ref = orc.forward(model, round_to(x, model["dtype"], torch), masks=masks)
    y = out_a.to_nchw()
    if model["head"] is not None:
        y = y[:, :, 0, 0]
    err = parity(y, ref, model["dtype"])
    print(f"resident model {mi}: rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


def test_imagenet_models_use_per_layer_schedule(fx):
    B, network, torch = fx
    model = synth.make_imagenet_basic_resnet(13, "bf16", (1, 1, 1, 1), 300, widths=(4, 8, 8, 12),
                                             size=32, classes=7)
    m, _ = network.build(network.optimise(model))
    assert m.num_launches == m.num_ops     # has a max-pool


@pytest.mark.parametrize("idx", range(5))
def test_baseline_config_full_batch(fx, idx):
    """The workload at its full batch size, launched the way bench.py launches it
    (HIP-graph replay on a side stream).  Configurations 0 - 3: the oracle computes
    EVERY image of the batch (tiles run across image boundaries and persistent
    workgroups walk ranges of tiles, so no image may go unchecked).  Configuration 4
    (256 images of the largest network): the oracle computes about fifteen images here, and
    test_config4_layer_shapes_at_full_batch covers every layer at the full batch."""
    B, network, torch = fx
    model, batch = synth.make_config(idx)
    dtype = model["dtype"]
    seed = synth.BASE_SEED + idx
    plan = network.optimise(model)
    m, _ = network.build(plan)
    x = synth.make_input(seed, batch, model["in_shape"])
    xd = B.DeviceTensor.from_nchw(x, B.DTYPES[dtype])
    s = torch.cuda.Stream()
    sp = B.C.c_void_p(s.cuda_stream)
    with torch.cuda.stream(s):
        out, ws = m.alloc(batch)
        out.data.fill_(float("nan"))
        s.synchronize()
        g = m.fupr_graph_create(xd, out, ws, sp)
        m.fupr_graph_launch(g, sp)
        s.synchronize()
    y = out.to_nchw()
    if model["head"] is not None:
        y = y[:, :, 0, 0]
    assert np.isfinite(y).all()
    masks = orc.select_masks(model)
    # (configuration 4: the first and last images, both sides of the boundary between the two
    # sub-batches and of each quarter, and a seeded handful in between)
    extra = [int(v) for v in np.random.default_rng(seed).integers(0, batch, 4)]
    sample = list(range(batch)) if idx < 4 else sorted(
        {0, 1, batch // 4 - 1, batch // 4, batch // 2 - 1, batch // 2, batch // 2 + 1, 3 * batch // 4 - 1,
         3 * batch // 4, batch - 2, batch - 1, *extra})
    print(f"config {idx}: batch {batch}, oracle on {len(sample)} images", flush=True)
    xr = round_to(x[sample], dtype, torch)
    worst = 0.0
    for at in range(0, len(sample), 16):       # 16 images per oracle pass bounds its memory
        ref = orc.forward(model, xr[at:at + 16], masks=masks)
        for j in range(ref.shape[0]):          # every image against its own maximum
            worst = max(worst, parity(y[sample[at + j]:sample[at + j] + 1], ref[j:j + 1], dtype,
                                      quiet=True))
    print(f"config {idx}: worst rel err over {len(sample)} images {worst:.3e}", flush=True)


def raw_layers(model):
    """site name -> (raw convolution, its batch norm, (block, conv) key or None)."""
    sites = {}
    if model["stem"] is not None:
        sites["stem"] = (model["stem"]["conv"], model["stem"]["bn"], None)
    for bi, blk in enumerate(model["blocks"]):
        for ci, (conv, bn) in enumerate(zip(blk["convs"], blk["bns"])):
            sites[f"b{bi}.conv{ci + 1}"] = (conv, bn, (bi, ci))
        if blk["shortcut"]["kind"] == "projection":
            sites[f"b{bi}.proj"] = (blk["shortcut"]["conv"], blk["shortcut"]["bn"], None)
    return sites


def test_config4_layer_shapes_at_full_batch(fx):
    """Every convolution of the largest workload (irregular channel counts, fp16)
    at its full batch of 256 images, each alone on seeded synthetic activations of
    its input shape: the device computes the whole layer, the oracle (raw weights,
    literal batch norm, removed filters and removed input channels as zeros) a
    sample of output pixels one by one - the corners of the first and last image,
    pixels either side of image boundaries, and seeded random ones."""
    B, network, torch = fx
    model, batch = synth.make_config(4)
    dtype = model["dtype"]
    dt = B.DTYPES[dtype]
    masks = orc.select_masks(model)
    plan = network.optimise(model, concat_projection=False)   # one operator per convolution site
    raw = raw_layers(model)
    rng = np.random.default_rng(synth.BASE_SEED + 4004)
    worst, done = 0.0, 0
    for L in plan["layers"]:
        if L.site == "fc":
            continue                      # a 1 x 1 image: covered at full batch by the network test
        conv, bn, key = raw[L.site]
        k_full, c_full, r, _ = conv["W"].shape
        stride, pad = conv["stride"], conv["pad"]
        in_keep = np.arange(c_full)
        if key is not None and (key[0], key[1] - 1) in masks:
            in_keep = np.flatnonzero(masks[(key[0], key[1] - 1)])
        out_keep = np.flatnonzero(masks[key]) if key in masks else np.arange(k_full)
        assert L.W.shape == (len(out_keep), len(in_keep), r, r), L.site
        # input extent from the site's place in the network
        h = {"stem": 224}.get(L.site)
        if h is None:
            bi = int(L.site[1:].split(".")[0])
            stage = 0 if bi < 3 else 1 if bi < 7 else 2 if bi < 13 else 3
            first = bi in (0, 3, 7, 13)
            out_h = 56 >> stage
            if L.site.endswith("conv3"):
                h = out_h
            elif L.site.endswith("conv2"):
                h = out_h * stride
            else:                          # conv1 and the projection read the block input
                h = out_h * (2 if first and stage > 0 else 1)
        p = (h + 2 * pad - r) // stride + 1
        c = len(in_keep)
        x = np.maximum(rng.standard_normal((batch, c, h, h), dtype=np.float32), 0.0)
        if L.site == "stem":
            x = rng.standard_normal((batch, c, h, h), dtype=np.float32)
        xd = B.DeviceTensor.from_nchw(x, dt)
        xr = round_to(x, dtype, torch) if x.size < (1 << 26) else None
        res_d = None
        if L.add:
            rs = np.maximum(rng.standard_normal((batch, len(out_keep), p, p), dtype=np.float32), 0.0)
            res_d = B.DeviceTensor.from_nchw(rs, dt)
        packed = B.upload_blob(B.fupr_pack(L.shape, L.W, L.bias, dt))
        yd = B.DeviceTensor.empty(batch, p, p, len(out_keep), dt)
        flags = (B.FUSE_RELU if L.relu else 0) | (B.FUSE_ADD if L.add else 0)
        print(f"{L.site}: {c} -> {len(out_keep)} {r}x{r}/{stride} on {batch}x{h}x{h}", flush=True)
        B.fupr_conv_fused(L.shape, xd, packed, (res_d, 1, 0) if L.add else None, flags, yd)
        torch.cuda.synchronize()
        # sampled output pixels (n, p, q)
        pts = [(0, 0, 0), (0, 0, p - 1), (0, p - 1, p - 1), (1, 0, 0), (batch // 2 - 1, p - 1, p - 1),
               (batch // 2, 0, 0), (batch - 1, p - 1, 0), (batch - 1, p - 1, p - 1)]
        pts += [(int(rng.integers(batch)), int(rng.integers(p)), int(rng.integers(p))) for _ in range(40)]
        crops = np.zeros((len(pts), c_full, r, r), dtype=np.float64)
        for j, (n, pp, qq) in enumerate(pts):
            for dr in range(r):
                for ds in range(r):
                    ih, iw = pp * stride + dr - pad, qq * stride + ds - pad
                    if 0 <= ih < h and 0 <= iw < h:
                        v = x[n, :, ih, iw] if xr is None else xr[n, :, ih, iw]
                        crops[j, in_keep, dr, ds] = round_to(v, dtype, torch) if xr is None else v
        ref = orc.batchnorm(orc.conv2d(crops, conv["W"], 1, 0), bn)[:, out_keep, 0, 0]
        got = np.stack([yd.data[n, pp, qq, :len(out_keep)].double().cpu().numpy() for n, pp, qq in pts])
        if L.add:
            ref = ref + np.stack([res_d.data[n, pp, qq, :len(out_keep)].double().cpu().numpy()
                                  for n, pp, qq in pts])
        if L.relu:
            ref = orc.relu(ref)
        worst = max(worst, parity(got, ref, dtype, quiet=True))
        done += 1
        del xd, yd, res_d, packed, x, xr
    print(f"config 4: {done} layers at batch {batch}, worst sampled rel err {worst:.3e}", flush=True)
    assert done == 53


def test_forward_is_deterministic_and_graph_replays(fx):
    B, network, torch = fx
    model = synth.make_cifar_resnet(21, "bf16", 3, 400)
    x = synth.make_input(21, 4, model["in_shape"])
    plan = network.optimise(model)
    m, _ = network.build(plan)
    xd = B.DeviceTensor.from_nchw(x, B.BF16)
    out, ws = m.alloc(4)
    m.fupr_forward(xd, out, ws)
    torch.cuda.synchronize()
    first = out.data.clone()
    m.fupr_forward(xd, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(first, out.data)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out2, ws2 = m.alloc(4)
        s.synchronize()
        g = m.fupr_graph_create(xd, out2, ws2, B.C.c_void_p(s.cuda_stream))
        for _ in range(3):
            out2.data.zero_()
            s.synchronize()
            m.fupr_graph_launch(g, B.C.c_void_p(s.cuda_stream))
            s.synchronize()
            assert torch.equal(first, out2.data)


def test_sub_batches_on_forked_streams_give_identical_results(fx):
    """Large batches run as sub-batches on streams that fork from and join the
    caller's stream; images are independent, so the result must not change by a
    bit, eagerly and from a replayed graph."""
    B, network, torch = fx
    model = synth.make_imagenet_basic_resnet(31, "bf16", (1, 1, 1, 1), 300, widths=(64, 16, 24, 40),
                                             size=64, classes=9)
    n = 26
    x = synth.make_input(31, n, model["in_shape"])
    m, _ = network.build(network.optimise(model))
    xd = B.DeviceTensor.from_nchw(x, B.BF16)
    out, ws = m.alloc(n)
    try:
        B.fupr_tuning_set("split", 1)
        m.fupr_forward(xd, out, ws)
        torch.cuda.synchronize()
        whole = out.data.clone()
        for parts in (2, 3):
            B.fupr_tuning_set("split", parts)
            print(f"sub-batches: {parts}", flush=True)
            out.data.zero_()
            m.fupr_forward(xd, out, ws)
            torch.cuda.synchronize()
            assert torch.equal(whole, out.data)
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                out2, ws2 = m.alloc(n)
                s.synchronize()
                g = m.fupr_graph_create(xd, out2, ws2, B.C.c_void_p(s.cuda_stream))
                for _ in range(3):
                    out2.data.zero_()
                    s.synchronize()
                    m.fupr_graph_launch(g, B.C.c_void_p(s.cuda_stream))
                    s.synchronize()
                    assert torch.equal(whole, out2.data)
    finally:
        B.fupr_tuning_set("split", None)


# ---- a block's pruned output filters: indexed update of the full-width stream --------------

SCATTER_CASES = [
    # name, N, C, H, W, kept filters, channels of y, R, relu
    ("3x3 C45 keep 45 of 64 56x56", 1, 45, 56, 56, 45, 64, 3, True),
    ("3x3 C90 keep 90 of 128 28x28 x3", 3, 90, 28, 28, 90, 128, 3, True),
    ("3x3 C180 keep 179 of 256 14x14", 2, 180, 14, 14, 179, 256, 3, True),
    ("3x3 C24 keep 5 of 24 ragged", 2, 24, 13, 11, 5, 24, 3, True),
    ("3x3 C16 keep 12 of 16 no relu", 2, 16, 32, 32, 12, 16, 3, False),
    ("3x3 C64 keep 100 of 100 7x7 x5", 5, 64, 7, 7, 100, 100, 3, True),
    ("3x3 C8 keep 3 of 10 general kernel", 1, 8, 9, 9, 3, 10, 3, True),
    ("3x3 C32 keep 5 of 8 one chunk", 2, 32, 10, 10, 5, 8, 3, True),
    ("3x3 C16 keep 20 of 1200 sparse", 1, 16, 6, 6, 20, 1200, 3, True),
    ("3x3 C64 keep 130 of 136 dense", 2, 64, 9, 9, 130, 136, 3, True),
    ("3x3 C48 keep 70 of 700 wide range", 1, 48, 8, 8, 70, 700, 3, False),
    ("1x1 C32 keep 180 of 256", 2, 32, 14, 14, 180, 256, 1, True),
    ("1x1 C64 keep 100 of 520 ragged", 3, 64, 7, 9, 100, 520, 1, True),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", SCATTER_CASES, ids=[c[0] for c in SCATTER_CASES])
def test_conv_scatter_site(fx, case, dtype):
    """The kept filters add into their channels of y in place; every other channel
    of y keeps its bits."""
    B, network, torch = fx
    name, n, c, h, w, k, width, r, relu = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    print(f"case={name} dtype={dtype}", flush=True)
    pad = r // 2
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = (rng.standard_normal((k, c, r, r)) * np.sqrt(2.0 / (c * r * r))).astype(np.float32)
    bn = {"gamma": rng.uniform(0.5, 1.5, k).astype(np.float32),
          "beta": (rng.standard_normal(k) * 0.1).astype(np.float32),
          "mean": (rng.standard_normal(k) * 0.1).astype(np.float32),
          "var": rng.uniform(0.5, 1.5, k).astype(np.float32), "eps": 1e-5}
    keep = np.sort(rng.choice(width, size=k, replace=False)).astype(np.int32)
    y0 = rng.standard_normal((n, width, h, w)).astype(np.float32)
    dt = B.DTYPES[dtype]

    y0r = round_to(y0, dtype, torch)
    upd = orc.add(orc.batchnorm(orc.conv2d(round_to(x, dtype, torch), wt, 1, pad), bn),
                  np.ascontiguousarray(y0r[:, keep]))
    if relu:
        upd = orc.relu(upd)

    sh = B.shape_of(wt, 1, pad)
    Wf, bf = B.fupr_fold(sh, wt, None, bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"],
                         B.FUSE_BN)
    packed = B.upload_blob(B.fupr_pack(sh, Wf, bf, dt))
    keep_d = torch.from_numpy(keep).cuda()
    xd = B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.from_nchw(y0, dt)
    B.fupr_conv_scatter_fused(sh, xd, packed, keep_d, B.FUSE_RELU if relu else 0, yd)
    torch.cuda.synchronize()
    got = yd.to_nchw()
    assert yd.padding_is_zero()
    rest = np.setdiff1d(np.arange(width), keep)
    assert np.array_equal(got[:, rest], y0r[:, rest])
    err = parity(got[:, keep], upd, dtype)
    print(f"  max-norm rel err {err:.3e}", flush=True)
    assert err <= TOL[dtype], (name, dtype, err)


def test_conv_scatter_random_shapes(fx):
    """Seeded random shapes and index lists (clustered and spread, few and many
    filter groups, ragged pixel counts): the chunk ownership of the 3 x 3 kernel's
    indexed epilogue must hold for every way the kept channels fall into chunks."""
    B, network, torch = fx
    rng = np.random.default_rng(20101616)
    worst = 0.0
    for case in range(24):
        r = 3 if case % 4 else 1
        width = int(rng.choice([16, 24, 40, 64, 72, 128, 200, 256, 520]))
        frac = float(rng.choice([0.15, 0.5, 0.7, 0.9, 1.0]))
        k = max(1, int(width * frac))
        c = int(rng.choice([16, 24, 32, 45, 64, 90]))
        h, w = int(rng.integers(5, 20)), int(rng.integers(5, 20))
        n = int(rng.integers(1, 4))
        dtype = "bf16" if case % 2 else "f16"
        if case % 3 == 0:      # clustered: a contiguous run of channels, then the rest spread
            start = int(rng.integers(0, width - k + 1))
            keep = np.arange(start, start + k)
        else:
            keep = np.sort(rng.choice(width, size=k, replace=False))
        keep = keep.astype(np.int32)
        print(f"case {case}: {r}x{r} C{c} keep {k} of {width}, {n}x{h}x{w} {dtype}", flush=True)
        pad = r // 2
        x = rng.standard_normal((n, c, h, w)).astype(np.float32)
        wt = (rng.standard_normal((k, c, r, r)) * np.sqrt(2.0 / (c * r * r))).astype(np.float32)
        bias = (rng.standard_normal(k) * 0.1).astype(np.float32)
        y0 = rng.standard_normal((n, width, h, w)).astype(np.float32)
        dt = B.DTYPES[dtype]
        y0r = round_to(y0, dtype, torch)
        conv = orc.conv2d(round_to(x, dtype, torch), round_to(wt, dtype, torch), 1, pad)
        upd = orc.relu(conv + bias.astype(np.float64)[None, :, None, None] + y0r[:, keep])
        sh = B.shape_of(wt, 1, pad)
        packed = B.upload_blob(B.fupr_pack(sh, wt, bias, dt))
        keep_d = torch.from_numpy(keep).cuda()
        xd = B.DeviceTensor.from_nchw(x, dt)
        yd = B.DeviceTensor.from_nchw(y0, dt)
        B.fupr_conv_scatter_fused(sh, xd, packed, keep_d, B.FUSE_RELU, yd)
        torch.cuda.synchronize()
        got = yd.to_nchw()
        rest = np.setdiff1d(np.arange(width), keep)
        assert np.array_equal(got[:, rest], y0r[:, rest]), case
        assert yd.padding_is_zero()
        err = parity(got[:, keep], upd, dtype, quiet=True)
        worst = max(worst, err)
        assert err <= TOL[dtype], (case, err)
    print(f"worst rel err {worst:.3e}", flush=True)


def test_conv_scatter_rejects_bad_calls(fx):
    B, network, torch = fx
    rng = np.random.default_rng(17)
    n, c, h, w, k, width = 2, 16, 12, 12, 6, 16
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = (rng.standard_normal((k, c, 3, 3)) * 0.1).astype(np.float32)
    bias = rng.standard_normal(k).astype(np.float32)
    y0 = rng.standard_normal((n, width, h, w)).astype(np.float32)
    keep = np.array([1, 2, 5, 9, 14, 15], dtype=np.int32)
    sh = B.shape_of(wt, 1, 1)
    dt = B.BF16
    packed = B.upload_blob(B.fupr_pack(sh, wt, bias, dt))
    keep_d = torch.from_numpy(keep).cuda()
    xd = B.DeviceTensor.from_nchw(x, dt)
    yd = B.DeviceTensor.from_nchw(y0, dt)
    before = yd.data.clone()

    def expect(code, fn):
        with pytest.raises(B.FuprError) as e:
            fn()
        assert e.value.status == code
        torch.cuda.synchronize()
        assert torch.equal(yd.data, before)

    narrow = B.DeviceTensor.from_nchw(y0[:, :4], dt)
    expect(B.ERR_SHAPE, lambda: B.fupr_conv_scatter_fused(sh, xd, packed, keep_d, 0, narrow))
    other = B.DeviceTensor.from_nchw(y0[:, :, :5], dt)
    expect(B.ERR_SHAPE, lambda: B.fupr_conv_scatter_fused(sh, xd, packed, keep_d, 0, other))
    expect(B.ERR_ARG, lambda: B.fupr_conv_scatter_fused(sh, xd, packed, keep_d, B.FUSE_ADD, yd))
    x32 = B.DeviceTensor.from_nchw(x, B.F32)
    y32 = B.DeviceTensor.from_nchw(y0, B.F32)
    p32 = B.upload_blob(B.fupr_pack(sh, wt, bias, B.F32))
    expect(B.ERR_DTYPE, lambda: B.fupr_conv_scatter_fused(sh, x32, p32, keep_d, 0, y32))
    xs, ys = xd.struct, yd.struct
    st = B._lib.fupr_conv_scatter_fused(B.C.byref(sh), B.C.byref(xs), B.C.c_void_p(packed.data_ptr()),
                                        None, 0, B.C.byref(ys), None)
    assert st == B.ERR_NULL


def stream_models():
    return [
        synth.make_cifar_resnet(42, "bf16", 2, 400, widths=(8, 16, 24), size=16, classes=5,
                                out_permille=300),
        synth.make_imagenet_basic_resnet(43, "f16", (2, 1, 2, 1), 300, widths=(8, 16, 16, 24), size=32,
                                         classes=7, out_permille=500),
        synth.make_imagenet_bottleneck_resnet(44, "bf16", (2, 2, 1, 1), 500, widths=(4, 4, 8, 8),
                                              size=32, classes=5, out_permille=300),
        synth.make_cifar_resnet(45, "bf16", 3, 300, out_permille=300),
    ]


@pytest.mark.parametrize("mi", range(4))
def test_network_with_pruned_output_filters(fx, mi):
    """Every block with an identity shortcut also loses output filters (the paper
    prunes all non-fused convolutions, Sec. V-A): against the zero-masked oracle."""
    B, network, torch = fx
    model = stream_models()[mi]
    x = synth.make_input(81, 3, model["in_shape"])
    masks = orc.select_masks(model)
    ref = orc.forward(model, round_to(x, model["dtype"], torch), masks=masks)
    plan, m, y = run_network(B, network, torch, model, x)
    assert set(plan["masks"]) == set(masks)
    n_stream = 0
    for key in masks:
        assert np.array_equal(plan["masks"][key], masks[key])
        assert np.array_equal(plan["keep_idx"][key], np.flatnonzero(masks[key]))
        n_stream += key[1] + 1 == len(model["blocks"][key[0]]["convs"])
    assert n_stream >= 2
    assert m.num_launches > 1     # kernels per operator (or pair), not the one-kernel schedule
    thin = [L for L in plan["layers"] if L.keep is not None]
    # 3 x 3 last convolutions run thin and add into their channels; 1 x 1 ones get zero rows back
    assert all(L.W.shape[2] == 3 for L in thin)
    assert bool(thin) == (model["blocks"][0]["kind"] == "basic")
    err = parity(y, ref, model["dtype"])
    print(f"model {mi} {model['name']} end-to-end rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]
    # the graph replays to the same bits (the updates are in place, the stream is rebuilt each pass)
    dt = B.DTYPES[model["dtype"]]
    xd = B.DeviceTensor.from_nchw(x, dt)
    out, ws = m.alloc(x.shape[0])
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = m.fupr_graph_create(xd, out, ws, B.C.c_void_p(stream.cuda_stream))
        for _ in range(3):
            out.data.zero_()
            stream.synchronize()
            m.fupr_graph_launch(g, B.C.c_void_p(stream.cuda_stream))
            stream.synchronize()
            assert np.array_equal(out.to_nchw()[:, :, 0, 0], y)


@pytest.mark.parametrize("name", ["resnet18", "resnet34"])
def test_paper_workload_with_pruned_output_filters(fx, name):
    B, network, torch = fx
    model = synth.make_paper_workload(name, 300, out_permille=300)
    x = synth.make_input(82, 2, model["in_shape"])
    masks = orc.select_masks(model)
    ref = orc.forward(model, round_to(x, model["dtype"], torch), masks=masks)
    plan, m, y = run_network(B, network, torch, model, x)
    kernels = [m.op_stats(2, i)["kernel"] for i, L in enumerate(m.sites) if L and L.endswith("conv2")]
    assert all(k.startswith("conv3x3p_") for k in kernels)
    err = parity(y, ref, model["dtype"])
    print(f"{model['name']}: rel err {err:.3e}", flush=True)
    assert err <= TOL[model["dtype"]]


@pytest.mark.parametrize("name,batch", [("resnet34", 64), ("resnet18", 192)])
def test_pruned_output_filters_full_batch_sampled(fx, name, batch):
    """The batch sizes bench.py uses, launched the way it launches them (HIP-graph
    replay on a side stream; 192 images run as two sub-batches on forked streams,
    each updating its own slice of the stream in place); the oracle computes three
    of the images."""
    B, network, torch = fx
    model = synth.make_paper_workload(name, 300, out_permille=300)
    dtype = model["dtype"]
    plan = network.optimise(model)
    m, _ = network.build(plan)
    x = synth.make_input(83, batch, model["in_shape"])
    xd = B.DeviceTensor.from_nchw(x, B.DTYPES[dtype])
    s = torch.cuda.Stream()
    sp = B.C.c_void_p(s.cuda_stream)
    with torch.cuda.stream(s):
        out, ws = m.alloc(batch)
        out.data.fill_(float("nan"))
        s.synchronize()
        g = m.fupr_graph_create(xd, out, ws, sp)
        for _ in range(2):
            m.fupr_graph_launch(g, sp)
            s.synchronize()
    y = out.to_nchw()[:, :, 0, 0]
    assert np.isfinite(y).all()
    masks = orc.select_masks(model)
    worst = 0.0
    for i in (0, batch // 2, batch - 1):
        ref = orc.forward(model, round_to(x[i:i + 1], dtype, torch), masks=masks)
        worst = max(worst, parity(y[i:i + 1], ref, dtype, quiet=True))
    print(f"{model['name']} batch {batch}: worst sampled rel err {worst:.3e}", flush=True)
    assert worst <= TOL[dtype]


def test_measuring_kernels(fx):
    """The copy copies; the MFMA loop reports its work and multiplies what it says
    (ones times ones, summed over 32 channels, iters times)."""
    B, network, torch = fx
    from paper_2010_16165_amd import measure as M
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    M.fupr_measure_copy(src, dst, src.numel())
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    with pytest.raises(RuntimeError):
        M.fupr_measure_copy(src, dst, 24)
    out = torch.zeros(4 * 256, dtype=torch.float32, device="cuda")
    for dt in (B.BF16, B.F16):
        for shape, chains, per_mfma in ((16, 16, 2 * 16 * 16 * 32), (32, 8, 2 * 32 * 32 * 16)):
            flops = M.fupr_measure_mfma(dt, shape, 3, 4, out)
            torch.cuda.synchronize()
            assert flops == 4 * 4 * 3 * chains * per_mfma   # workgroups, waves, iterations, chains
            assert torch.isfinite(out).all() and float(out.abs().max()) > 0
    with pytest.raises(RuntimeError):
        M.fupr_measure_mfma(B.F32, 16, 3, 4, out)
    with pytest.raises(RuntimeError):
        M.fupr_measure_mfma(B.BF16, 8, 3, 4, out)


def test_timed_forward_and_stats(fx):
    B, network, torch = fx
    model = synth.make_cifar_resnet(22, "bf16", 2, 400)
    x = synth.make_input(22, 2, model["in_shape"])
    plan = network.optimise(model)
    m, sites = network.build(plan)
    xd = B.DeviceTensor.from_nchw(x, B.BF16)
    out, ws = m.alloc(2)
    ms = m.fupr_forward_timed(xd, out, ws)
    assert ms.shape == (m.num_ops,) and ms[0] > 0 and (ms[m.num_launches:] == 0).all()
    total = sum(m.op_stats(2, i)["flops"] for i in range(m.num_ops))
    assert m.launch_stats(2, 0)["flops"] == total and m.launch_stats(2, 0)["kernel"] == "resident_network"
    m.set_schedule(B.SCHEDULE_PER_LAYER)
    ms = m.fupr_forward_timed(xd, out, ws)
    assert (ms > 0).all()
    st = m.op_stats(2, 0)
    assert st["flops"] == 2.0 * 3 * 9 * 16 * 2 * 32 * 32 and st["kernel"].startswith("conv16")


# ---- error paths on device calls (nothing is launched) ------------------------------

def test_device_call_errors(fx):
    B, network, torch = fx
    dt = B.BF16
    wt = np.zeros((16, 16, 3, 3), dtype=np.float32)
    sh = B.shape_of(wt, 1, 1)
    packed = B.upload_blob(B.fupr_pack(sh, wt, None, dt))
    x = B.DeviceTensor.empty(1, 8, 8, 16, dt)
    y = B.DeviceTensor.empty(1, 8, 8, 16, dt)
    y.data.fill_(5.0)

    def expect(code, fn):
        with pytest.raises(B.FuprError) as e:
            fn()
        assert e.value.status == code

    bad_y = B.DeviceTensor.empty(1, 7, 8, 16, dt)
    expect(B.ERR_SHAPE, lambda: B.fupr_conv_fused(sh, x, packed, None, 0, bad_y))
    expect(B.ERR_NULL, lambda: B.fupr_conv_fused(sh, x, packed, None, B.FUSE_ADD, y))
    expect(B.ERR_ARG, lambda: B.fupr_conv_fused(sh, x, packed, (x, 1, 0), 0, y))
    expect(B.ERR_ARG, lambda: B.fupr_conv_fused(sh, x, packed, None, 64, y))
    expect(B.ERR_DTYPE, lambda: B.fupr_conv_fused(sh, x, packed, None, 0,
                                                  B.DeviceTensor.empty(1, 8, 8, 16, B.F16)))
    expect(B.ERR_ARG, lambda: B.fupr_conv_fused(sh, x, packed, None, 0, x))
    torch.cuda.synchronize()
    assert bool((y.data == 5.0).all())
