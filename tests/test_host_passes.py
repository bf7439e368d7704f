"""CPU tests of the library's host side: the C-ABI surface, batch-norm merge,
filter selection, filter removal, packing, model planning and error paths.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth
from oracle import reference as orc
from paper_2010_16165_amd import binding as B, network

RNG = np.random.default_rng(3)
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def rand_bn(k):
    f = lambda a: np.asarray(a, dtype=np.float32)
    return {"gamma": f(RNG.uniform(0.5, 1.5, k)), "beta": f(RNG.standard_normal(k) * 0.1),
            "mean": f(RNG.standard_normal(k) * 0.1), "var": f(RNG.uniform(0.5, 1.5, k)), "eps": 1e-5}


# ---- C ABI surface ------------------------------------------------------------

def declared_in(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    return set(re.findall(r"\b(fupr_[a-z_0-9]+)\s*\(", header))


def test_library_exports_every_declared_symbol():
    declared = declared_in("fupr.h")
    assert len(declared) >= 20
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)


def test_measuring_library_exports_every_declared_symbol():
    """The measuring kernels live in a library of their own, apart from the product's."""
    from paper_2010_16165_amd import measure as M
    declared = declared_in("fupr_measure.h")
    assert declared == set(M.SIGNATURES) == {"fupr_measure_mfma", "fupr_measure_copy"}
    lib = C.CDLL(M.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    product = C.CDLL(B.LIB_PATH)
    assert not any(hasattr(product, name) for name in declared)


def test_library_owns_no_device_memory_or_stream():
    """Every device buffer and stream is the caller's: the product sources call no
    allocating, copying or stream-creating runtime routine."""
    csrc = os.path.join(ROOT, "paper_2010_16165_amd", "csrc")
    banned = re.compile(r"\bhip(Malloc\w*|Free\w*|Memcpy\w*|Memset\w*|StreamCreate\w*|HostMalloc|ExtMalloc\w*)\s*\(")
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        text = re.sub(r"//.*", "", text)
        hits = banned.findall(text)
        assert not hits, (name, hits)


def build_host_model(plan, base):
    return network.build(plan, base_address=base)


def test_tuning_switches():
    B.fupr_tuning_set("patch_tile", 4)
    B.fupr_tuning_set("patch_tile", None)
    B.fupr_tuning_set("conv_tile", "conv16t_64x16")
    B.fupr_tuning_set("conv_tile", "")
    for name in ("pipe_tile", "pipe_order", "stream_tile", "stream_blocks", "pair_filters", "split",
                 "conv_patch", "conv1x1_stream", "conv1x1_pipe", "conv1x1_fuse", "res_item", "debug"):
        B.fupr_tuning_set(name, 1)
        B.fupr_tuning_set(name, None)
    for gone in ("block_fuse", "block_tile"):      # switches of a kernel that was never built
        with pytest.raises(B.FuprError):
            B.fupr_tuning_set(gone, 1)
    with pytest.raises(B.FuprError) as e:
        B.fupr_tuning_set("no_such_switch", 1)
    assert e.value.status == B.ERR_ARG
    with pytest.raises(B.FuprError) as e:
        B.fupr_tuning_set("split", "9" * 200)
    assert e.value.status == B.ERR_ARG
    assert B._lib.fupr_tuning_set(None, None) == B.ERR_NULL


def test_one_kernel_table_is_the_callers():
    """The one-kernel schedule's table is written on the host for a device address
    the caller names; without one the model runs a kernel per operator."""
    model = synth.make_cifar_resnet(5, "bf16", 2, 400)
    plan = network.optimise(model)
    # host-only: made-up 256-byte aligned "device" addresses, nothing is dereferenced here
    base = 1 << 20
    m, _ = build_host_model(plan, base)
    nbytes = B._lib.fupr_model_table_bytes(m._h)
    assert nbytes > 0 and nbytes % 256 == 0
    assert m.num_launches == m.num_ops            # no table yet: per operator
    img_a = np.zeros(nbytes, np.uint8)
    img_b = np.zeros(nbytes, np.uint8)
    st = B._lib.fupr_model_table_write(m._h, C.c_void_p(1 << 30), img_a.ctypes.data_as(C.c_void_p))
    assert st == B.FUPR_OK
    st = B._lib.fupr_model_table_write(m._h, C.c_void_p((1 << 30) + 4096), img_b.ctypes.data_as(C.c_void_p))
    assert st == B.FUPR_OK
    assert not np.array_equal(img_a, img_b)       # the image holds addresses inside itself
    assert B._lib.fupr_model_table_write(m._h, C.c_void_p((1 << 30) + 8), img_a.ctypes.data_as(C.c_void_p)) == B.ERR_ALIGN
    assert B._lib.fupr_model_table_write(m._h, None, img_a.ctypes.data_as(C.c_void_p)) == B.ERR_NULL
    assert B._lib.fupr_model_set_table(m._h, C.c_void_p(1 << 30)) == B.FUPR_OK
    assert m.num_launches == 1
    assert B._lib.fupr_model_set_table(m._h, None) == B.FUPR_OK
    assert m.num_launches == m.num_ops
    # a network with a max-pool has no such table
    big = synth.make_imagenet_basic_resnet(13, "bf16", (1, 1, 1, 1), 300, widths=(4, 8, 8, 12), size=32, classes=7)
    mb, _ = build_host_model(network.optimise(big), base)
    assert B._lib.fupr_model_table_bytes(mb._h) == 0
    assert B._lib.fupr_model_set_table(mb._h, C.c_void_p(1 << 30)) == B.ERR_ARG
    assert B._lib.fupr_model_table_bytes(None) == 0


def test_side_streams_argument_checks():
    model = synth.make_cifar_resnet(5, "bf16", 1, 400)
    m, _ = build_host_model(network.optimise(model), 1 << 20)
    arr = (C.c_void_p * 4)(None, None, None, None)
    assert B._lib.fupr_model_set_side_streams(m._h, 0, None) == B.FUPR_OK
    assert B._lib.fupr_model_set_side_streams(m._h, 1, None) == B.ERR_NULL
    assert B._lib.fupr_model_set_side_streams(m._h, 1, arr) == B.ERR_NULL      # NULL stream
    assert B._lib.fupr_model_set_side_streams(m._h, 4, arr) == B.ERR_ARG
    assert B._lib.fupr_model_set_side_streams(m._h, -1, arr) == B.ERR_ARG
    assert B._lib.fupr_model_set_side_streams(None, 0, None) == B.ERR_NULL


def test_status_strings():
    for code in range(0, -12, -1):
        assert B.status_str(code) not in ("", "unknown status")
    assert B.status_str(-99) == "unknown status"


# ---- fold (Eq. 3-5 and the merge) -------------------------------------------------

def test_fold_matches_closed_form():
    w = RNG.standard_normal((6, 5, 3, 3)).astype(np.float32)
    bn = rand_bn(6)
    sh = B.shape_of(w, 1, 1)
    wf, bf = B.fupr_fold(sh, w, None, bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"],
                         B.FUSE_BN)
    wo, bo = orc.fold(w, bn)
    assert wf.dtype == np.float32 and bf.dtype == np.float32
    np.testing.assert_allclose(wf, wo, rtol=2 ** -23)
    np.testing.assert_allclose(bf, bo, rtol=2 ** -22, atol=1e-9)


def test_fold_then_conv_equals_conv_then_bn():
    x = RNG.standard_normal((2, 5, 7, 7))
    w = RNG.standard_normal((6, 5, 3, 3)).astype(np.float32)
    bn = rand_bn(6)
    cb = RNG.standard_normal(6).astype(np.float32)
    sh = B.shape_of(w, 1, 1)
    wf, bf = B.fupr_fold(sh, w, cb, bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"],
                         B.FUSE_BN)
    ref = orc.batchnorm(orc.conv2d(x, w, 1, 1) + cb[None, :, None, None].astype(np.float64), bn)
    got = orc.conv2d(x, wf, 1, 1) + bf[None, :, None, None].astype(np.float64)
    assert np.abs(got - ref).max() / np.abs(ref).max() <= 1e-5


def test_fold_identity_special_case_is_exact():
    k = 4
    var = RNG.uniform(0.5, 1.5, k).astype(np.float32)
    mean = RNG.standard_normal(k).astype(np.float32)
    # gamma = sqrt(var + eps) in double, eps = 0 so that omega is exactly 1 for perfect squares
    var = (np.arange(1, k + 1, dtype=np.float32)) ** 2
    gamma = np.arange(1, k + 1, dtype=np.float32)
    w = RNG.standard_normal((k, 3, 3, 3)).astype(np.float32)
    sh = B.shape_of(w, 1, 1)
    wf, bf = B.fupr_fold(sh, w, None, gamma, mean, mean, var, 0.0, B.FUSE_BN)
    assert np.array_equal(wf, w) and np.all(bf == 0)


def test_fold_without_bn_flag_copies():
    w = RNG.standard_normal((3, 2, 1, 1)).astype(np.float32)
    b = RNG.standard_normal(3).astype(np.float32)
    sh = B.shape_of(w, 1, 0)
    wf, bf = B.fupr_fold(sh, w, b, None, None, None, None, 1e-5, 0)
    assert np.array_equal(wf, w) and np.array_equal(bf, b)
    wf, bf = B.fupr_fold(sh, w, None, None, None, None, None, 1e-5, B.FUSE_RELU)
    assert np.all(bf == 0)


def expect(code, fn):
    with pytest.raises(B.FuprError) as e:
        fn()
    assert e.value.status == code, (e.value.status, code)


def test_fold_errors_leave_outputs_untouched():
    w = np.ones((2, 2, 1, 1), dtype=np.float32)
    bn = rand_bn(2)
    sh = B.shape_of(w, 1, 0)
    bad_var = np.array([1.0, -1.0], dtype=np.float32)
    expect(B.ERR_BN_VAR, lambda: B.fupr_fold(sh, w, None, bn["gamma"], bn["beta"], bn["mean"],
                                             bad_var, 1e-5, B.FUSE_BN))
    expect(B.ERR_BN_VAR, lambda: B.fupr_fold(sh, w, None, bn["gamma"], bn["beta"], bn["mean"],
                                             np.array([1.0, np.inf], dtype=np.float32), 1e-5,
                                             B.FUSE_BN))
    expect(B.ERR_NULL, lambda: B.fupr_fold(sh, w, None, None, bn["beta"], bn["mean"], bn["var"],
                                           1e-5, B.FUSE_BN))
    expect(B.ERR_ARG, lambda: B.fupr_fold(sh, w, None, bn["gamma"], bn["beta"], bn["mean"],
                                          bn["var"], 1e-5, 128))
    expect(B.ERR_SHAPE, lambda: B.fupr_fold(B.conv_shape(0, 2, 1, 1, 1, 0), w, None, bn["gamma"],
                                            bn["beta"], bn["mean"], bn["var"], 1e-5, B.FUSE_BN))
    # raw call: outputs keep their sentinel on error
    wout = np.full(4, 9.0, dtype=np.float32)
    bout = np.full(2, 9.0, dtype=np.float32)
    F = B._F
    st = B._lib.fupr_fold(C.byref(sh), w.ctypes.data_as(F), None, bn["gamma"].ctypes.data_as(F),
                          bn["beta"].ctypes.data_as(F), bn["mean"].ctypes.data_as(F),
                          bad_var.ctypes.data_as(F), C.c_float(1e-5), B.FUSE_BN,
                          wout.ctypes.data_as(F), bout.ctypes.data_as(F))
    assert st == B.ERR_BN_VAR and np.all(wout == 9.0) and np.all(bout == 9.0)


# ---- filter selection ------------------------------------------------------------------

@pytest.mark.parametrize("n,permille", [(16, 250), (16, 400), (32, 400), (64, 400), (64, 300),
                                        (128, 300), (256, 300), (512, 300), (64, 500), (4, 1000),
                                        (7, 0), (1, 999), (2048, 137)])
def test_prune_count_matches_oracle(n, permille):
    assert B.fupr_prune_count(n, permille) == orc.prune_count(n, permille)


def test_prune_count_errors():
    expect(B.ERR_ARG, lambda: B.fupr_prune_count(0, 100))
    expect(B.ERR_ARG, lambda: B.fupr_prune_count(8, 1001))
    expect(B.ERR_ARG, lambda: B.fupr_prune_count(8, -1))


@pytest.mark.parametrize("norm", [1, 2])
def test_select_filters_bit_exact_vs_oracle(norm):
    for k, c, r in [(16, 16, 3), (64, 3, 7), (39, 64, 3), (256, 64, 1), (5, 1, 1)]:
        w = RNG.standard_normal((k, c, r, r)).astype(np.float32)
        for n_prune in (0, 1, k // 3, k - 1):
            got = B.fupr_select_filters(B.shape_of(w, 1, 0), w, norm, n_prune)
            assert np.array_equal(got, orc.select_mask(w, n_prune, norm))
            assert int(got.sum()) == k - n_prune


def test_select_filters_tie_rule_and_norm_choice():
    w = np.ones((6, 2, 3, 3), dtype=np.float32)
    assert list(B.fupr_select_filters(B.shape_of(w, 1, 1), w, 1, 2)) == [0, 0, 1, 1, 1, 1]
    w = np.zeros((2, 4, 1, 1), dtype=np.float32)
    w[0, :, 0, 0] = 1
    w[1, 0, 0, 0] = 3
    sh = B.shape_of(w, 1, 0)
    assert list(B.fupr_select_filters(sh, w, 1, 1)) == [1, 0]
    assert list(B.fupr_select_filters(sh, w, 2, 1)) == [0, 1]
    expect(B.ERR_ARG, lambda: B.fupr_select_filters(sh, w, 3, 1))
    expect(B.ERR_ARG, lambda: B.fupr_select_filters(sh, w, 1, 2))
    expect(B.ERR_ARG, lambda: B.fupr_select_filters(sh, w, 1, -1))


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_masks_of_baseline_configs_match_oracle(idx):
    model, _ = synth.make_config(idx)
    plan = network.optimise(model)
    masks = orc.select_masks(model)
    assert set(plan["masks"]) == set(masks) and masks
    for key, m in masks.items():
        assert np.array_equal(plan["masks"][key], m)
        assert np.array_equal(plan["keep_idx"][key], np.flatnonzero(m))
        assert plan["keep_idx"][key].dtype == np.int32


# ---- filter removal -----------------------------------------------------------------------

def test_prune_is_an_exact_gather():
    wp = RNG.standard_normal((9, 4, 3, 3)).astype(np.float32)
    bp = RNG.standard_normal(9).astype(np.float32)
    wc1 = RNG.standard_normal((7, 9, 3, 3)).astype(np.float32)
    wc2 = RNG.standard_normal((5, 9, 1, 1)).astype(np.float32)
    mask = np.array([1, 0, 1, 1, 0, 0, 1, 0, 1], dtype=np.uint8)
    keep, wpo, bpo, (w1o, w2o) = B.fupr_prune(B.shape_of(wp, 1, 1), wp, bp, mask,
                                              [B.shape_of(wc1, 1, 1), B.shape_of(wc2, 2, 0)],
                                              [wc1, wc2])
    idx = [0, 2, 3, 6, 8]
    assert list(keep) == idx
    # gather written out by hand
    for j, k in enumerate(idx):
        assert wpo[j].tobytes() == wp[k].tobytes() and bpo[j] == bp[k]
        for f in range(7):
            assert w1o[f, j].tobytes() == wc1[f, k].tobytes()
        for f in range(5):
            assert w2o[f, j].tobytes() == wc2[f, k].tobytes()
    assert wpo.shape == (5, 4, 3, 3) and w1o.shape == (7, 5, 3, 3) and w2o.shape == (5, 5, 1, 1)


def test_prune_without_bias_or_consumers():
    wp = RNG.standard_normal((4, 2, 1, 1)).astype(np.float32)
    keep, wpo, bpo, rest = B.fupr_prune(B.shape_of(wp, 1, 0), wp, None, [0, 1, 1, 0], [], [])
    assert list(keep) == [1, 2] and bpo is None and rest == [] and np.array_equal(wpo, wp[1:3])


def test_prune_and_fold_commute():
    """Per-filter scaling commutes with the gather: bit-exact either way round."""
    w1 = RNG.standard_normal((8, 3, 3, 3)).astype(np.float32)
    w2 = RNG.standard_normal((6, 8, 3, 3)).astype(np.float32)
    bn1, bn2 = rand_bn(8), rand_bn(6)
    s1, s2 = B.shape_of(w1, 1, 1), B.shape_of(w2, 1, 1)
    mask = B.fupr_select_filters(s1, w1, 1, 3)
    fold = lambda sh, w, bn: B.fupr_fold(sh, w, None, bn["gamma"], bn["beta"], bn["mean"],
                                         bn["var"], bn["eps"], B.FUSE_BN)
    # fold, then prune
    w1f, b1f = fold(s1, w1, bn1)
    w2f, b2f = fold(s2, w2, bn2)
    _, a1, ab1, (a2,) = B.fupr_prune(s1, w1f, b1f, mask, [s2], [w2f])
    # prune, then fold
    keep, p1, _, (p2,) = B.fupr_prune(s1, w1, None, mask, [s2], [w2])
    bn1k = {k: (v[keep] if k != "eps" else v) for k, v in bn1.items()}
    c1, cb1 = fold(B.shape_of(p1, 1, 1), p1, bn1k)
    c2, _ = fold(B.shape_of(p2, 1, 1), p2, bn2)
    assert np.array_equal(a1, c1) and np.array_equal(ab1, cb1) and np.array_equal(a2, c2)


def test_prune_errors():
    wp = np.ones((4, 2, 1, 1), dtype=np.float32)
    sh = B.shape_of(wp, 1, 0)
    wc = np.ones((3, 4, 1, 1), dtype=np.float32)
    expect(B.ERR_MASK_EMPTY, lambda: B.fupr_prune(sh, wp, None, [0, 0, 0, 0], [], []))
    expect(B.ERR_ARG, lambda: B.fupr_prune(sh, wp, None, [1, 2, 0, 0], [], []))
    bad = B.conv_shape(3, 5, 1, 1, 1, 0)     # consumer C != producer K
    expect(B.ERR_SHAPE, lambda: B.fupr_prune(sh, wp, None, [1, 1, 0, 0], [bad], [wc]))


def test_library_compaction_equals_oracle_extraction():
    """The thinner model the library builds is the oracle's `extract` of the
    merged weights, filter for filter."""
    model = synth.make_imagenet_bottleneck_resnet(14, "bf16", (2, 1, 1, 1), 500, widths=(4, 4, 8, 8),
                                                  size=32, classes=5)
    plan = network.optimise(model, concat_projection=False)
    thin = orc.extract(model, orc.select_masks(model))
    by_site = {L.site: L for L in plan["layers"]}
    for bi, blk in enumerate(thin["blocks"]):
        for ci, (conv, bn) in enumerate(zip(blk["convs"], blk["bns"])):
            L = by_site[f"b{bi}.conv{ci + 1}"]
            wo, bo = orc.fold(conv["W"], bn)
            assert L.W.shape == wo.shape
            np.testing.assert_allclose(L.W, wo, rtol=2 ** -23)
            np.testing.assert_allclose(L.bias, bo, rtol=2 ** -22, atol=1e-9)


# ---- packing ---------------------------------------------------------------------------------

def bf16_bits_rne(a):
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


@pytest.mark.parametrize("k,c,r", [(10, 16, 3), (16, 10, 3), (64, 3, 7), (39, 64, 3), (1000, 20, 1),
                                   (1, 1, 1)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_pack_16bit_layout(k, c, r, dtype):
    w = RNG.standard_normal((k, c, r, r)).astype(np.float32)
    b = RNG.standard_normal(k).astype(np.float32)
    sh = B.shape_of(w, 1, r // 2)
    blob = B.fupr_pack(sh, w, b, B.DTYPES[dtype])
    kp, cp = (k + 15) // 16 * 16, (c + 7) // 8 * 8
    nchunk = r * r * cp // 8
    nchunk_pad = (nchunk + 3) // 4 * 4
    woff = (kp * 4 + 255) // 256 * 256
    assert len(blob) == (woff + nchunk_pad * kp * 16 + 255) // 256 * 256 == B.fupr_packed_bytes(
        sh, B.DTYPES[dtype])
    bias = blob[:kp * 4].view(np.float32)
    assert np.array_equal(bias[:k], b) and np.all(bias[k:] == 0)
    wt = blob[woff:woff + nchunk_pad * kp * 16].view(np.uint16).reshape(nchunk_pad, kp, 8)
    expect_bits = np.zeros((nchunk_pad, kp, 8), dtype=np.uint16)
    bits = bf16_bits_rne(w) if dtype == "bf16" else w.astype(np.float16).view(np.uint16)
    for rr in range(r):
        for ss in range(r):
            for cc in range(c):
                expect_bits[(rr * r + ss) * (cp // 8) + cc // 8, :k, cc % 8] = bits[:, cc, rr, ss]
    assert np.array_equal(wt, expect_bits)


def test_pack_16bit_rounding_edge_cases():
    vals = np.array([1.0, 1.00390625, 1.01171875, 65519.9, 65520.0, 1e-8, 5.96e-8, 6.1e-5, -0.0,
                     3.0e-5, np.inf, 70000.0], dtype=np.float32)
    w = np.zeros((1, 16, 1, 1), dtype=np.float32)
    w[0, :len(vals), 0, 0] = vals
    sh = B.shape_of(w, 1, 0)
    for dtype in ("bf16", "f16"):
        blob = B.fupr_pack(sh, w, None, B.DTYPES[dtype])
        wt = blob[256:256 + 4 * 16 * 16].view(np.uint16).reshape(4, 16, 8)
        got = np.concatenate([wt[0, 0], wt[1, 0]])
        with np.errstate(over="ignore"):
            want = bf16_bits_rne(w[0, :, 0, 0]) if dtype == "bf16" else \
                w[0, :, 0, 0].astype(np.float16).view(np.uint16)
        assert np.array_equal(got, want), dtype


def test_pack_f32_layout():
    k, c, r = 10, 6, 3
    w = RNG.standard_normal((k, c, r, r)).astype(np.float32)
    sh = B.shape_of(w, 1, 1)
    blob = B.fupr_pack(sh, w, None, B.F32)
    kp, cp = 12, 8
    assert len(blob) == 256 + (r * r * cp * kp * 4 + 255) // 256 * 256
    assert np.all(blob[:kp * 4].view(np.float32) == 0)
    wt = blob[256:256 + r * r * cp * kp * 4].view(np.float32).reshape(r * r, cp, kp)
    want = np.zeros((r * r, cp, kp), dtype=np.float32)
    want[:, :c, :k] = w.transpose(2, 3, 1, 0).reshape(r * r, c, k)
    assert np.array_equal(wt, want)


def test_pack_errors():
    assert B.fupr_packed_bytes(B.conv_shape(0, 1, 1, 1, 1, 0), B.BF16) == 0
    assert B.fupr_packed_bytes(B.conv_shape(1, 1, 1, 1, 1, 0), 7) == 0
    w = np.zeros((1, 1, 1, 1), dtype=np.float32)
    st = B._lib.fupr_pack(C.byref(B.conv_shape(1, 1, 1, 1, 1, 0)), w.ctypes.data_as(B._F), None, 7,
                          C.c_void_p(w.ctypes.data))
    assert st == B.ERR_DTYPE
    st = B._lib.fupr_pack(C.byref(B.conv_shape(1, 1, 1, 1, 1, 0)), None, None, B.BF16,
                          C.c_void_p(w.ctypes.data))
    assert st == B.ERR_NULL


# ---- model planning (host only; device pointers are never dereferenced) -----------------------

def fake_ops(specs):
    """specs: (kind, in, res, K, C, R, stride, pad, epilogue, rss)"""
    ops = []
    for kind, tin, res, k, c, r, st, pd, epi, rss in specs:
        ops.append(B.OpDesc(kind, tin, res, B.conv_shape(k, c, r, r, st, pd), 0x1000, epi, rss, 0))
    return ops


def test_model_plan_shares_buffers_and_reports_shapes():
    ops = fake_ops([
        (B.OP_CONV, 0, -1, 16, 3, 3, 1, 1, B.FUSE_RELU, 1),                  # t1 16x32x32
        (B.OP_CONV, 1, -1, 10, 16, 3, 1, 1, B.FUSE_RELU, 1),                 # t2
        (B.OP_CONV, 2, 1, 16, 10, 3, 1, 1, B.FUSE_RELU | B.FUSE_ADD, 1),     # t3 (+t1)
        (B.OP_CONV, 3, -1, 20, 16, 3, 2, 1, B.FUSE_RELU, 1),                 # t4 20x16x16
        (B.OP_CONV, 4, 3, 32, 20, 3, 1, 1, B.FUSE_RELU | B.FUSE_ADD, 2),     # t5 32x16x16 (+t3 ::2)
        (B.OP_AVGPOOL, 5, -1, 1, 1, 1, 1, 0, 0, 1),
        (B.OP_CONV, 6, -1, 10, 32, 1, 1, 0, 0, 1),
    ])
    m = B.Model(B.BF16, (3, 32, 32), ops, None)
    assert m.num_ops == 7
    t = m.output_shape(5)
    assert (t.N, t.H, t.W, t.C, t.c_stride) == (5, 1, 1, 10, 16)
    # three live 16-channel 32x32 tensors at most -> three buffers of 32 KB per image
    assert m.workspace_bytes(1) == 3 * 32 * 32 * 16 * 2
    assert m.workspace_bytes(4) == 4 * m.workspace_bytes(1)
    s = m.op_stats(2, 2)
    assert s["flops"] == 2.0 * 10 * 9 * 16 * 2 * 1024
    assert s["bytes"] == 2 * (2 * 1024 * 10 + 2 * 1024 * 16 + 2 * 1024 * 16 + 16 * 10 * 9) + 4 * 16
    assert s["kernel"].startswith("conv")


def test_kernel_selection_per_layer_class():
    """Which kernel an operator launches is decided on the host from its shape
    alone: every layer class of the ImageNet workloads must get its own kernel."""
    ops = fake_ops([
        (B.OP_CONV, 0, -1, 64, 3, 7, 2, 3, B.FUSE_RELU, 1),                   # t1 64 x 112 x 112
        (B.OP_MAXPOOL, 1, -1, 1, 1, 3, 2, 1, 0, 1),                           # t2 64 x 56 x 56
        (B.OP_CONV, 2, -1, 45, 64, 3, 1, 1, B.FUSE_RELU, 1),                  # t3
        (B.OP_CONV, 3, 2, 64, 45, 3, 1, 1, B.FUSE_RELU | B.FUSE_ADD, 1),      # t4
        (B.OP_CONV, 4, -1, 256, 64, 1, 1, 0, 0, 1),                           # t5 256 x 56 x 56
        (B.OP_CONV, 5, -1, 32, 256, 1, 1, 0, B.FUSE_RELU, 1),                 # t6
        (B.OP_CONV, 6, -1, 90, 32, 3, 2, 1, B.FUSE_RELU, 1),                  # t7 90 x 28 x 28
        (B.OP_CONV, 7, -1, 1024, 90, 1, 2, 0, 0, 1),                          # t8 1024 x 14 x 14
        (B.OP_CONV, 8, -1, 128, 1024, 1, 1, 0, B.FUSE_RELU, 1),               # t9
    ])
    m = B.Model(B.BF16, (3, 224, 224), ops, None)
    names = [m.op_stats(64, i)["kernel"] for i in range(m.num_ops)]
    assert names[2].startswith("conv3x3p_") and names[3].startswith("conv3x3p_")
    assert names[4].startswith("conv1x1s_") and names[5].startswith("conv1x1s_")
    assert names[6].startswith("conv16t_")        # stride 2 at 56 x 56: the general kernel
    assert names[8].startswith("conv1x1p_")       # 1024 channels: filters do not fit in LDS
    # the stem convolution and the max-pool behind it are one launch, and so are
    # the 64 -> 256 and 256 -> 32 1 x 1 convolutions (the second from the first's registers)
    assert m.num_launches == m.num_ops - 2
    pair = m.launch_stats(64, 3)
    a, b = m.op_stats(64, 4), m.op_stats(64, 5)
    assert pair["kernel"] == "conv1x1s_256f+conv1x1" and pair["flops"] == a["flops"] + b["flops"]
    assert pair["bytes"] == a["bytes"] + b["bytes"] - 2 * 64 * 56 * 56 * 256
    first = m.launch_stats(64, 0)
    assert first["kernel"] == "stem7x7_maxpool"
    conv, pool = m.op_stats(64, 0), m.op_stats(64, 1)
    mid = 2 * 64 * 112 * 112 * 64
    assert first["flops"] == conv["flops"] and first["bytes"] == conv["bytes"] + pool["bytes"] - 2 * mid
    m.set_schedule(B.SCHEDULE_PER_LAYER)
    assert m.num_launches == m.num_ops and m.launch_stats(64, 0)["kernel"].startswith("conv16t_")


def test_model_create_errors():
    ok = (B.OP_CONV, 0, -1, 16, 3, 3, 1, 1, B.FUSE_RELU, 1)
    cases = [
        ([(B.OP_CONV, 0, -1, 16, 4, 3, 1, 1, 0, 1)], B.ERR_SHAPE),             # C mismatch
        ([ok, (B.OP_CONV, 2, -1, 16, 16, 3, 1, 1, 0, 1)], B.ERR_ARG),          # reads a later tensor
        ([ok, (B.OP_CONV, 1, 0, 16, 16, 3, 1, 1, 0, 1)], B.ERR_ARG),           # res without ADD
        ([ok, (B.OP_CONV, 1, -1, 16, 16, 3, 1, 1, B.FUSE_ADD, 1)], B.ERR_ARG),  # ADD without res
        ([ok, (B.OP_CONV, 1, 0, 16, 16, 3, 2, 1, B.FUSE_ADD, 3)], B.ERR_SHAPE),  # residual too small
        ([ok, (7, 1, -1, 1, 1, 1, 1, 0, 0, 1)], B.ERR_ARG),                    # unknown kind
        ([ok, (B.OP_MAXPOOL, 1, -1, 1, 1, 3, 2, 3, 0, 1)], B.ERR_ARG),         # pad >= window
        ([(B.OP_CONV, 0, -1, 16, 3, 40, 1, 1, 0, 1)], B.ERR_SHAPE),            # window larger than image
    ]
    for specs, code in cases:
        expect(code, lambda: B.Model(B.BF16, (3, 32, 32), fake_ops(specs), None))
    expect(B.ERR_DTYPE, lambda: B.Model(5, (3, 32, 32), fake_ops([ok]), None))
    bad = fake_ops([ok])
    bad[0].packed = None
    expect(B.ERR_NULL, lambda: B.Model(B.BF16, (3, 32, 32), bad, None))


def test_baseline_config_graphs_have_expected_launch_counts():
    want = {0: 2, 1: 56, 2: 21, 3: 54, 4: 54}
    for idx, n in want.items():
        model, _ = synth.make_config(idx)
        plan = network.optimise(model, concat_projection=False)
        assert len(plan["layers"]) == n
        # a bottleneck block's projection shortcut is part of its last convolution by default
        plan = network.optimise(model)
        assert len(plan["layers"]) == n - (4 if idx >= 3 else 0)
        assert sum(L.cat_stride > 0 for L in plan["layers"]) == (4 if idx >= 3 else 0)


def test_largest_workload_pairs_its_first_stage_output_with_the_next_convolution():
    """The launch list of the largest workload: stem + pool, three pairs of 1 x 1 convolutions in
    the first stage (the third with the 90-filter first convolution of the next stage), 48
    launches for 52 operators; with pairs limited to 64 second filters it has one more."""
    model, batch = synth.make_config(4)
    plan = network.optimise(model)
    m, _ = build_host_model(plan, 1 << 20)
    assert (m.num_ops, m.num_launches) == (52, 48)
    kernels = [m.launch_stats(batch, i)["kernel"] for i in range(m.num_launches)]
    assert kernels.count("conv1x1s_256f+conv1x1") == 3 and kernels[0] == "stem7x7_maxpool"
    B.fupr_tuning_set("pair_filters", 64)
    try:
        m2, _ = build_host_model(plan, 1 << 20)
        assert m2.num_launches == 49
    finally:
        B.fupr_tuning_set("pair_filters", None)


# ---- a block's pruned output filters (Alg. 1 on every non-fused operator, Sec. V-A) ---------

def scatter_ops(keep=0x2000, **change):
    """stem, conv1, conv2 whose 11 kept filters add into the stem's 16 channels, head."""
    specs = [
        (B.OP_CONV, 0, -1, 16, 3, 3, 1, 1, B.FUSE_RELU, 1),                          # t1 16 x 32 x 32
        (B.OP_CONV, 1, -1, 10, 16, 3, 1, 1, B.FUSE_RELU, 1),                         # t2
        (B.OP_CONV, 2, 1, 11, 10, 3, 1, 1, B.FUSE_RELU | B.FUSE_ADD | B.FUSE_SCATTER, 1),  # t3 = t1 updated
        (B.OP_AVGPOOL, 3, -1, 1, 1, 1, 1, 0, 0, 1),
        (B.OP_CONV, 4, -1, 10, 16, 1, 1, 0, 0, 1),
    ]
    for i, spec in change.get("specs", {}).items():
        specs[i] = spec
    ops = fake_ops(specs)
    ops[2].keep_idx = keep
    return ops


def test_model_plan_updates_the_stream_in_place():
    m = B.Model(B.BF16, (3, 32, 32), scatter_ops(), None)
    # t1 and t2 only: the update needs no buffer of its own
    assert m.workspace_bytes(1) == 2 * 32 * 32 * 16 * 2
    s = m.op_stats(2, 2)
    assert s["K"] == 11 and s["C"] == 10
    assert s["flops"] == 2.0 * 10 * 9 * 11 * 2 * 1024
    # input once, 11 channels of the stream read and written, parameters, index list
    assert s["bytes"] == 2 * (2 * 1024 * 10 + 2 * 2 * 1024 * 11 + 11 * 10 * 9) + 8 * 11
    assert s["kernel"].startswith("conv3x3p_") or s["kernel"].startswith("conv16t_")
    t = m.output_shape(3)
    assert (t.C, t.c_stride) == (10, 16)
    # no one-kernel schedule with such an operator
    assert m.num_launches == m.num_ops


def test_model_create_errors_of_in_place_updates():
    S = B.FUSE_RELU | B.FUSE_ADD | B.FUSE_SCATTER
    expect(B.ERR_NULL, lambda: B.Model(B.BF16, (3, 32, 32), scatter_ops(keep=None), None))
    cases = [
        ({2: (B.OP_CONV, 2, -1, 11, 10, 3, 1, 1, B.FUSE_RELU | B.FUSE_SCATTER, 1)}, B.ERR_ARG),  # no tensor
        ({2: (B.OP_CONV, 2, 1, 17, 10, 3, 1, 1, S, 1)}, B.ERR_SHAPE),          # more filters than channels
        ({2: (B.OP_CONV, 2, 1, 11, 10, 3, 2, 1, S, 1)}, B.ERR_SHAPE),          # other extent
        ({2: (B.OP_CONV, 2, 1, 11, 10, 3, 1, 1, S, 2)}, B.ERR_ARG),            # strided shortcut
        ({1: (B.OP_CONV, 0, -1, 10, 3, 3, 1, 1, B.FUSE_RELU, 1),
          2: (B.OP_CONV, 2, 0, 3, 10, 3, 1, 1, S, 1)}, B.ERR_ARG),             # the network input
        ({3: (B.OP_CONV, 1, -1, 10, 16, 1, 1, 0, 0, 1),
          4: (B.OP_CONV, 3, -1, 10, 16, 1, 1, 0, 0, 1)}, B.ERR_ARG),           # old number read later
    ]
    for change, code in cases:
        expect(code, lambda: B.Model(B.BF16, (3, 32, 32), scatter_ops(specs=change), None))
    expect(B.ERR_DTYPE, lambda: B.Model(B.F32, (3, 32, 32), scatter_ops(), None))
    last = scatter_ops()[:3]
    expect(B.ERR_ARG, lambda: B.Model(B.BF16, (3, 32, 32), last, None))       # the network's last operator
    plain = fake_ops([(B.OP_CONV, 0, -1, 16, 3, 3, 1, 1, B.FUSE_RELU, 1)])
    plain[0].keep_idx = 0x2000
    expect(B.ERR_ARG, lambda: B.Model(B.BF16, (3, 32, 32), plain, None))      # index list without the flag


def test_output_filter_plan_matches_oracle():
    """Masks and kept-filter lists of the blocks' last convolutions are the oracle's,
    the compacted weights are its extraction, and only identity blocks take part."""
    model = synth.make_imagenet_basic_resnet(23, "bf16", (2, 1, 2, 1), 300, widths=(4, 8, 8, 12),
                                             size=32, classes=7, out_permille=500)
    plan = network.optimise(model)
    masks = orc.select_masks(model)
    assert set(plan["masks"]) == set(masks)
    thin = orc.extract(model, masks)
    by_site = {L.site: L for L in plan["layers"]}
    n_stream = 0
    for bi, blk in enumerate(thin["blocks"]):
        L = by_site[f"b{bi}.conv2"]
        if "stream_keep" in blk:
            assert blk["shortcut"]["kind"] == "identity"
            assert np.array_equal(L.keep, blk["stream_keep"]) and L.keep.dtype == np.int32
            assert np.array_equal(plan["masks"][(bi, 1)], masks[(bi, 1)])
            n_stream += 1
        else:
            assert L.keep is None
        wo, bo = orc.fold(blk["convs"][1]["W"], blk["bns"][1])
        assert L.W.shape == wo.shape
        np.testing.assert_allclose(L.W, wo, rtol=2 ** -23)
        np.testing.assert_allclose(L.bias, bo, rtol=2 ** -22, atol=1e-9)
    assert n_stream == 3
    proj = synth.make_imagenet_basic_resnet(26, "bf16", (1, 1), 300, widths=(4, 8), size=16, classes=3)
    proj["blocks"][1]["prune_permille"][1] = 300
    with pytest.raises(ValueError):
        network.optimise(proj)


# ---- aggressive fusion (Sec. IV-B) -------------------------------------------------

def fusible_blocks():
    a = synth.make_cifar_resnet(21, "bf16", 2, 400, widths=(4, 8, 12), size=12, classes=5)
    b = synth.make_imagenet_basic_resnet(22, "bf16", (1, 2, 1, 1), 300, widths=(4, 8, 8, 12), size=32,
                                         classes=7)
    return a["blocks"] + b["blocks"]


def test_xconv_fuse_matches_oracle_construction():
    kinds = set()
    for blk in fusible_blocks():
        kinds.add(blk["shortcut"]["kind"])
        got = network._aggressive(blk)
        ref = orc.aggressive_fuse_block(blk)
        for ci in range(2):
            a, b = got["convs"][ci]["W"], ref["convs"][ci]["W"]
            assert a.dtype == np.float32 and a.shape == b.shape
            np.testing.assert_allclose(a, b, rtol=2e-7, atol=0)
            assert np.array_equal(a == 0, b == 0)
            for key in ("gamma", "beta", "mean", "var"):
                np.testing.assert_allclose(got["bns"][ci][key], ref["bns"][ci][key], rtol=2e-7, atol=1e-9)
        n, m = got["convs"][0]["W"].shape[0], ref["original_filters"][0]
        assert got["prune_counts"] == [n - m, 0]
    assert kinds == {"identity", "optionA", "projection"}


def test_aggressive_plan_selects_the_oracles_filters():
    model = synth.make_imagenet_basic_resnet(22, "bf16", (1, 2, 1, 1), 300, widths=(4, 8, 8, 12),
                                             size=32, classes=7)
    plan = network.optimise(model, aggressive=True)
    masks = orc.select_masks(orc.aggressive_fuse(model))
    assert set(plan["masks"]) == set(masks)
    for key in masks:
        assert np.array_equal(plan["masks"][key], masks[key])
    assert not any(L.add for L in plan["layers"])
    unpruned = network.optimise(model, aggressive=True, prune_fused=False)
    assert not unpruned["masks"]
    k, c = model["blocks"][0]["convs"][0]["W"].shape[:2]
    by_site = {L.site: L for L in unpruned["layers"]}
    assert by_site["b0.conv1"].W.shape == (k + c, c, 3, 3)
    assert by_site["b0.conv2"].W.shape == (k, k + c, 3, 3)


def test_partially_fused_plan_selects_the_oracles_filters():
    """Fusion option x/n: the blocks of the first x stages go through fupr_xconv_fuse
    and lose n - m filters, the rest are pruned at their rate; masks equal the oracle's."""
    model = synth.make_imagenet_basic_resnet(23, "bf16", (1, 2, 1, 1), 300, widths=(4, 8, 8, 12),
                                             size=32, classes=7)
    for stages in (0, 1, 3, 4):
        plan = network.optimise(model, aggressive=True, fuse_stages=stages)
        masks = orc.select_masks(orc.aggressive_fuse(model, stages=stages))
        assert set(plan["masks"]) == set(masks)
        for key in masks:
            assert np.array_equal(plan["masks"][key], masks[key])
        fused = sum(b["stage"] < stages for b in model["blocks"])
        assert sum(L.add for L in plan["layers"]) == len(model["blocks"]) - fused


def test_proj_concat_is_the_filterwise_concatenation():
    """conv(h, W) + conv_p(x, Wp) = conv([h ; x], [W | Wp]) (Sec. IV-B-1): exact copies of
    both weight sets with zeros between them up to a multiple of 64 channels, biases added;
    the oracle's two convolutions and addition equal its one convolution of the concatenation."""
    rng = np.random.default_rng(12)
    k, c1, c2 = 20, 20, 24
    assert B.CAT_ALIGN == 64
    W = rng.standard_normal((k, c1, 1, 1)).astype(np.float32)
    Wp = rng.standard_normal((k, c2, 1, 1)).astype(np.float32)
    b, bp = rng.standard_normal(k).astype(np.float32), rng.standard_normal(k).astype(np.float32)
    sh, shp = B.shape_of(W, 1, 0), B.shape_of(Wp, 2, 0)
    out, Wc, bc = B.fupr_proj_concat(sh, W, b, shp, Wp, bp)
    assert (out.K, out.C, out.R, out.S, out.stride, out.pad) == (k, 64 + c2, 1, 1, 1, 0)
    assert np.array_equal(Wc[:, :c1], W) and not Wc[:, c1:64].any() and np.array_equal(Wc[:, 64:], Wp)
    assert np.array_equal(bc, b + bp)
    h = rng.standard_normal((2, c1, 5, 6))
    x = rng.standard_normal((2, c2, 10, 12))
    two = orc.add(orc.conv2d(h, W, 1, 0), orc.conv2d(x, Wp, 2, 0))
    cat = np.concatenate([h, np.zeros((2, 64 - c1, 5, 6)), x[:, :, ::2, ::2]], axis=1)
    one = orc.conv2d(cat, Wc, 1, 0)
    np.testing.assert_allclose(one, two, rtol=1e-12, atol=1e-12)
    # errors: a 3 x 3 last convolution, different filter counts, a strided last convolution
    W3 = np.zeros((k, c1, 3, 3), np.float32)
    for bad_last, bad_proj in ((B.shape_of(W3, 1, 1), shp), (sh, B.conv_shape(k + 1, c2, 1, 1, 2, 0)),
                               (B.conv_shape(k, c1, 1, 1, 2, 0), shp)):
        with pytest.raises(B.FuprError) as e:
            B.fupr_proj_concat(bad_last, W3 if bad_last.R == 3 else W, b, bad_proj,
                               np.zeros((bad_proj.K, c2, 1, 1), np.float32), None)
        assert e.value.status == B.ERR_SHAPE


def test_model_accepts_a_two_input_convolution():
    def ops(in2=1, stride=2, c=64 + 16, epi=B.FUSE_RELU | B.FUSE_CAT):
        o = fake_ops([
            (B.OP_CONV, 0, -1, 16, 3, 3, 1, 1, B.FUSE_RELU, 1),      # t1 16 x 32 x 32
            (B.OP_CONV, 1, -1, 12, 16, 3, 2, 1, B.FUSE_RELU, 1),     # t2 12 x 16 x 16
            (B.OP_CONV, 2, -1, 40, c, 1, 1, 0, epi, 1),              # t3 = conv([t2 ; t1 at stride 2])
        ])
        o[2].in2, o[2].in2_spatial_stride = in2, stride
        return o
    m = B.Model(B.BF16, (3, 32, 32), ops(), None)
    s = m.op_stats(2, 2)
    assert s["flops"] == 2.0 * (12 + 16) * 40 * 2 * 256 and s["C"] == 28
    # t1 stays alive until the last operator: three buffers... t1 and t2 only (t3 is the output)
    assert m.workspace_bytes(1) == (32 * 32 * 16 + 16 * 16 * 16) * 2
    expect(B.ERR_SHAPE, lambda: B.Model(B.BF16, (3, 32, 32), ops(c=32 + 16), None))   # split not at 64
    expect(B.ERR_ARG, lambda: B.Model(B.BF16, (3, 32, 32), ops(in2=3), None))
    expect(B.ERR_ARG, lambda: B.Model(B.BF16, (3, 32, 32), ops(stride=3), None))
    B.Model(B.BF16, (3, 32, 32), ops(in2=0, c=64 + 3, stride=1), None)      # any earlier tensor large enough
    expect(B.ERR_SHAPE, lambda: B.Model(B.BF16, (3, 32, 32), ops(in2=2, c=64 + 12, stride=2), None))  # too small
    expect(B.ERR_DTYPE, lambda: B.Model(B.F32, (3, 32, 32), ops(), None))


def test_xconv_fuse_errors():
    blk = fusible_blocks()[0]
    c1, c2 = blk["convs"]
    b1, b2 = blk["bns"]
    # a zero scale after conv2 cannot be inverted
    bad = dict(b2)
    g = b2["gamma"].copy()
    g[1] = 0.0
    bad["gamma"] = g
    with pytest.raises(B.FuprError) as e:
        B.fupr_xconv_fuse(c1, b1, c2, bad, B.SHORTCUT_IDENTITY)
    assert e.value.status == B.ERR_BN_SCALE
    # var + eps must be positive
    bad = dict(b2)
    bad["var"] = -np.ones_like(b2["var"])
    with pytest.raises(B.FuprError) as e:
        B.fupr_xconv_fuse(c1, b1, c2, bad, B.SHORTCUT_IDENTITY)
    assert e.value.status == B.ERR_BN_VAR
    # unknown shortcut kind, projection without its convolution, mismatched conv2
    with pytest.raises(B.FuprError) as e:
        B.fupr_xconv_fuse(c1, b1, c2, b2, 7)
    assert e.value.status == B.ERR_ARG
    with pytest.raises(B.FuprError) as e:
        B.fupr_xconv_fuse(c1, b1, c2, b2, B.SHORTCUT_PROJECTION)
    assert e.value.status == B.ERR_NULL
    wrong = {"W": np.zeros((4, 5, 3, 3), np.float32), "stride": 1, "pad": 1}
    with pytest.raises(B.FuprError) as e:
        B.fupr_xconv_fuse(c1, b1, wrong, b2, B.SHORTCUT_IDENTITY)
    assert e.value.status == B.ERR_SHAPE
    even = {"W": np.zeros((4, 4, 2, 2), np.float32), "stride": 1, "pad": 1}
    with pytest.raises(B.FuprError) as e:
        B.fupr_xconv_fuse(even, b1, even, b2, B.SHORTCUT_IDENTITY)
    assert e.value.status == B.ERR_SHAPE


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more must end with a message, not a run."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
