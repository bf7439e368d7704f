"""Pins of the CPU oracle against things other than itself: closed forms,
special cases stated by the paper, brute force, and library routines."""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import reference as orc

RNG = np.random.default_rng(7)


def brute_conv(x, w, stride, pad):
    """Seven nested loops, python floats (double)."""
    n_, c_, h_, w_ = x.shape
    k_, _, r_, s_ = w.shape
    p_ = (h_ + 2 * pad - r_) // stride + 1
    q_ = (w_ + 2 * pad - s_) // stride + 1
    y = np.zeros((n_, k_, p_, q_))
    for n, k, p, q in itertools.product(range(n_), range(k_), range(p_), range(q_)):
        acc = 0.0
        for c, r, s in itertools.product(range(c_), range(r_), range(s_)):
            ih, iw = p * stride + r - pad, q * stride + s - pad
            if 0 <= ih < h_ and 0 <= iw < w_:
                acc += float(x[n, c, ih, iw]) * float(w[k, c, r, s])
        y[n, k, p, q] = acc
    return y


# ---- convolution ----------------------------------------------------------

def identity_weights(c, r=3):
    """W~ of Sec. IV-B-1: x = xconv(x, W~)."""
    w = np.zeros((c, c, r, r))
    for i in range(c):
        w[i, i, r // 2, r // 2] = 1.0
    return w


@pytest.mark.parametrize("c,h,w", [(1, 5, 5), (3, 8, 6), (16, 9, 9)])
def test_identity_kernel_copies_input(c, h, w):
    x = RNG.standard_normal((2, c, h, w))
    y = orc.conv2d(x, identity_weights(c), 1, 1)
    assert np.array_equal(y, x)


def test_identity_kernel_stride2_subsamples():
    x = RNG.standard_normal((2, 4, 9, 8))
    y = orc.conv2d(x, identity_weights(4), 2, 1)
    assert np.array_equal(y, x[:, :, ::2, ::2])


def test_1x1_is_per_pixel_matrix_product():
    x = RNG.standard_normal((2, 5, 4, 6))
    w = RNG.standard_normal((7, 5, 1, 1))
    y = orc.conv2d(x, w, 1, 0)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
def test_1x1_equals_zero_padded_3x3(stride):
    """A 1x1 conv padded with zeros to 3x3 gives the same output (Sec. IV-B-1)."""
    x = RNG.standard_normal((2, 5, 8, 8))
    w1 = RNG.standard_normal((6, 5, 1, 1))
    w3 = np.zeros((6, 5, 3, 3))
    w3[:, :, 1, 1] = w1[:, :, 0, 0]
    assert np.array_equal(orc.conv2d(x, w1, stride, 0), orc.conv2d(x, w3, stride, 1))


def test_all_ones_counts_taps():
    c = 3
    x = np.ones((1, c, 6, 7))
    w = np.ones((2, c, 3, 3))
    y = orc.conv2d(x, w, 1, 1)
    assert y.shape == (1, 2, 6, 7)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * c)
    assert np.all(y[:, :, 0, 1:-1] == 6 * c) and np.all(y[:, :, 1:-1, 0] == 6 * c)
    for p, q in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(y[:, :, p, q] == 4 * c)


@pytest.mark.parametrize("c,k,r,stride,pad,h,w", [
    (1, 1, 3, 1, 1, 5, 4), (3, 5, 3, 2, 1, 7, 6), (5, 3, 1, 2, 0, 6, 6),
    (12, 17, 3, 1, 1, 4, 5), (17, 12, 1, 1, 0, 3, 3), (3, 4, 7, 2, 3, 11, 9),
    (2, 3, 3, 1, 0, 5, 5),
])
def test_conv_matches_brute_force(c, k, r, stride, pad, h, w):
    x = RNG.standard_normal((2, c, h, w))
    wt = RNG.standard_normal((k, c, r, r))
    np.testing.assert_allclose(orc.conv2d(x, wt, stride, pad), brute_conv(x, wt, stride, pad),
                               rtol=1e-13, atol=1e-13)


def test_conv_is_not_symmetric_in_r_s_or_flipped():
    """A single off-centre tap tells cross-correlation from flipped convolution
    and r from s."""
    x = np.zeros((1, 1, 5, 5))
    x[0, 0, 2, 2] = 1.0
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 0, 1] = 1.0      # r = 0 (up), s = 1 (centre column)
    y = orc.conv2d(x, w, 1, 1)
    # y[p,q] = x[p + r - 1, q + s - 1] = x[p - 1, q]  ->  the impulse moves DOWN one row
    expect = np.zeros((1, 1, 5, 5))
    expect[0, 0, 3, 2] = 1.0
    assert np.array_equal(y, expect)


@pytest.mark.parametrize("c,k,r,stride,pad", [(8, 12, 3, 1, 1), (16, 10, 3, 2, 1), (3, 16, 7, 2, 3),
                                              (24, 9, 1, 2, 0)])
def test_conv_matches_library(c, k, r, stride, pad):
    x = RNG.standard_normal((3, c, 14, 13))
    wt = RNG.standard_normal((k, c, r, r))
    ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(wt), stride=stride, padding=pad).numpy()
    np.testing.assert_allclose(orc.conv2d(x, wt, stride, pad), ref, rtol=1e-12, atol=1e-12)


# ---- batch norm, fold ----------------------------------------------------

def test_batchnorm_hand_values():
    bn = {"gamma": np.array([2.0, 0.5]), "beta": np.array([1.0, -1.0]),
          "mean": np.array([3.0, 0.0]), "var": np.array([4.0 - 1e-5, 0.25 - 1e-5]), "eps": 1e-5}
    x = np.zeros((1, 2, 1, 2))
    x[0, 0] = [5.0, 3.0]
    x[0, 1] = [1.0, -2.0]
    y = orc.batchnorm(x, bn)
    np.testing.assert_allclose(y[0, 0, 0], [2 * (5 - 3) / 2 + 1, 1.0], rtol=1e-15)
    np.testing.assert_allclose(y[0, 1, 0], [0.5 * 1 / 0.5 - 1, 0.5 * -2 / 0.5 - 1], rtol=1e-15)


def _rand_bn(k):
    return {"gamma": RNG.uniform(0.5, 1.5, k), "beta": RNG.standard_normal(k) * 0.1,
            "mean": RNG.standard_normal(k) * 0.1, "var": RNG.uniform(0.5, 1.5, k), "eps": 1e-5}


def test_batchnorm_matches_library():
    x = RNG.standard_normal((2, 6, 5, 4))
    bn = _rand_bn(6)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    ref = F.batch_norm(t(x), t(bn["mean"]), t(bn["var"]), t(bn["gamma"]), t(bn["beta"]),
                       training=False, eps=bn["eps"]).numpy()
    np.testing.assert_allclose(orc.batchnorm(x, bn), ref, rtol=1e-12, atol=1e-12)


def test_fold_is_affine_form_of_bn():
    """BN(x) = omega x + lambda (Eq. 3-5): merged conv equals conv then literal bn."""
    x = RNG.standard_normal((2, 5, 7, 7))
    w = RNG.standard_normal((6, 5, 3, 3))
    bn = _rand_bn(6)
    wf, bf = orc.fold(w, bn)
    a = orc.batchnorm(orc.conv2d(x, w, 1, 1), bn)
    b = orc.conv2d(x, wf, 1, 1) + bf[None, :, None, None]
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)


def test_fold_identity_special_case():
    """gamma = sqrt(var + eps), beta = mean  =>  omega = 1, lambda = 0."""
    k = 4
    var = RNG.uniform(0.5, 1.5, k)
    mean = RNG.standard_normal(k)
    bn = {"gamma": np.sqrt(var + 1e-5), "beta": mean.copy(), "mean": mean, "var": var, "eps": 1e-5}
    w = RNG.standard_normal((k, 3, 3, 3))
    wf, bf = orc.fold(w, bn)
    np.testing.assert_allclose(wf, w, rtol=1e-15)
    np.testing.assert_allclose(bf, 0, atol=1e-15)


def test_fold_with_conv_bias():
    w = RNG.standard_normal((3, 2, 1, 1))
    bn = _rand_bn(3)
    b = RNG.standard_normal(3)
    x = RNG.standard_normal((1, 2, 3, 3))
    wf, bf = orc.fold(w, bn, b)
    a = orc.batchnorm(orc.conv2d(x, w, 1, 0) + b[None, :, None, None], bn)
    np.testing.assert_allclose(orc.conv2d(x, wf, 1, 0) + bf[None, :, None, None], a, rtol=1e-12,
                               atol=1e-12)


# ---- scalar operators and the rest of Table II ----------------------------

def test_relu_add():
    a = np.array([[-1.0, 0.0, 2.5, -0.0]])
    assert np.array_equal(orc.relu(a), [[0.0, 0.0, 2.5, 0.0]])
    assert np.array_equal(orc.add(a, 2 * a), 3 * a)


def test_shortcut_subsample_pad():
    x = RNG.standard_normal((2, 3, 8, 8))
    y = orc.shortcut_subsample_pad(x, 6, 2)
    assert y.shape == (2, 6, 4, 4)
    assert np.array_equal(y[:, :3], x[:, :, ::2, ::2])
    assert np.all(y[:, 3:] == 0)


def test_maxpool_library_and_border():
    x = RNG.standard_normal((2, 3, 9, 10))
    ref = F.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(orc.maxpool(x, 3, 2, 1), ref)
    # all-negative input: out-of-range taps must be ignored, not read as zero
    xn = -np.abs(x) - 1.0
    assert np.all(orc.maxpool(xn, 3, 2, 1) < 0)


def test_global_mean_and_fc():
    x = RNG.standard_normal((3, 4, 5, 6))
    np.testing.assert_allclose(orc.global_mean(x), x.mean(axis=(2, 3)), rtol=1e-13)
    v = RNG.standard_normal((3, 7))
    w = RNG.standard_normal((5, 7))
    b = RNG.standard_normal(5)
    np.testing.assert_allclose(orc.fc(v, w, b), v @ w.T + b, rtol=1e-13, atol=1e-13)


# ---- filter selection ------------------------------------------------------

def test_norm_closed_forms():
    w = np.zeros((3, 2, 1, 2))
    w[0] = [[[3, -4]], [[0, 0]]]       # l1 7, l2 5
    w[1] = [[[1, 1]], [[1, -1]]]       # l1 4, l2 2
    w[2] = [[[0, 0]], [[0, 6]]]        # l1 6, l2 6
    np.testing.assert_allclose(orc.filter_norms(w, 1), [7, 4, 6])
    np.testing.assert_allclose(orc.filter_norms(w, 2), [5, 2, 6])


def test_l1_and_l2_pick_different_filters():
    w = np.zeros((2, 4, 1, 1))
    w[0, :, 0, 0] = [1, 1, 1, 1]       # l1 4, l2 2
    w[1, :, 0, 0] = [3, 0, 0, 0]       # l1 3, l2 3
    assert list(orc.select_mask(w, 1, norm=1)) == [1, 0]
    assert list(orc.select_mask(w, 1, norm=2)) == [0, 1]


def test_tie_rule_prunes_lower_index_first():
    w = np.ones((6, 2, 3, 3))
    assert list(orc.select_mask(w, 2, norm=1)) == [0, 0, 1, 1, 1, 1]


def test_known_order():
    w = np.zeros((5, 1, 1, 1))
    w[:, 0, 0, 0] = [0.5, -0.1, 0.3, -0.9, 0.2]
    assert list(orc.select_mask(w, 2, norm=1)) == [1, 0, 1, 1, 0]
    assert list(orc.select_mask(w, 0, norm=1)) == [1] * 5


@pytest.mark.parametrize("n,permille,kept", [(16, 250, 12), (16, 400, 10), (32, 400, 20),
                                             (64, 400, 39), (64, 300, 45), (128, 300, 90),
                                             (256, 300, 180), (512, 300, 359), (64, 500, 32),
                                             (4, 1000, 1)])
def test_prune_count_closed_form(n, permille, kept):
    """A non-fused operator loses floor(p_phi * n) filters (Alg. 1)."""
    assert n - orc.prune_count(n, permille) == kept


def test_config0_mask_cardinality():
    model, _ = synth.make_config(0)
    masks = orc.select_masks(model)
    assert list(masks) == [(0, 0)]
    assert int(masks[(0, 0)].sum()) == 12 and masks[(0, 0)].dtype == np.uint8


# ---- networks --------------------------------------------------------------

def torch_forward(model, x):
    """The same wiring written with library operators (double precision)."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))

    def cb(h, conv, bn):
        h = F.conv2d(h, t(conv["W"]), stride=conv["stride"], padding=conv["pad"])
        return F.batch_norm(h, t(bn["mean"]), t(bn["var"]), t(bn["gamma"]), t(bn["beta"]),
                            training=False, eps=bn["eps"])

    h = t(x)
    if model["stem"] is not None:
        h = F.relu(cb(h, model["stem"]["conv"], model["stem"]["bn"]))
        if model["stem"]["maxpool"] is not None:
            h = F.max_pool2d(h, *model["stem"]["maxpool"])
    for blk in model["blocks"]:
        sc = blk["shortcut"]
        if sc["kind"] == "identity":
            short = h
        elif sc["kind"] == "optionA":
            k = blk["convs"][-1]["W"].shape[0]
            short = F.pad(h[:, :, ::2, ::2], (0, 0, 0, 0, 0, k - h.shape[1]))
        else:
            short = cb(h, sc["conv"], sc["bn"])
        g = h
        for conv, bn in zip(blk["convs"][:-1], blk["bns"][:-1]):
            g = F.relu(cb(g, conv, bn))
        h = F.relu(cb(g, blk["convs"][-1], blk["bns"][-1]) + short)
    if model["head"] is None:
        return h.numpy()
    h = F.adaptive_avg_pool2d(h, 1).flatten(1)
    return F.linear(h, t(model["head"]["fc_W"]), t(model["head"]["fc_b"])).numpy()


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
def test_network_matches_library_wiring(mi):
    model = small_models()[mi]
    x = synth.make_input(99, 2, model["in_shape"])
    y = orc.forward(model, x)
    ref = torch_forward(model, x)
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-10 * np.abs(ref).max())


@pytest.mark.parametrize("mi", range(5))
def test_merged_network_equals_unmerged(mi):
    """Merging bn into the conv before it is an equivalence (Sec. VI-B-3)."""
    model = small_models()[mi]
    x = synth.make_input(98, 2, model["in_shape"])
    a = orc.forward(model, x)
    b = orc.forward(model, x, merged=True)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-10 * np.abs(a).max())


@pytest.mark.parametrize("mi", range(5))
def test_removed_filters_equal_zeroed_filters(mi):
    """Removing the masked filters (Alg. 1, last step) gives bit-for-bit the
    output of the full-width network with those filters zeroed."""
    model = small_models()[mi]
    x = synth.make_input(97, 2, model["in_shape"])
    masks = orc.select_masks(model)
    assert masks
    zeroed = orc.forward(model, x, masks=masks)
    thin = orc.extract(model, masks)
    for (bi, ci), m in masks.items():
        assert thin["blocks"][bi]["convs"][ci]["W"].shape[0] == int(m.sum())
        assert thin["blocks"][bi]["convs"][ci + 1]["W"].shape[1] == int(m.sum())
    removed = orc.forward(thin, x)
    assert np.array_equal(zeroed, removed)
    # and pruning changes the result (the masks are not vacuous)
    assert not np.array_equal(zeroed, orc.forward(model, x))


def test_pruned_network_matches_library_with_zeroed_filters():
    model = small_models()[1]
    x = synth.make_input(96, 2, model["in_shape"])
    masks = orc.select_masks(model)
    y = orc.forward(model, x, masks=masks)
    ref = torch_forward(orc.zero_masked(model, masks), x)
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-10 * np.abs(ref).max())


# ---- output filters of a block (Sec. V-A: all non-fused convolutions are pruned) -----

def stream_models():
    return [
        synth.make_block_model(21, "bf16", 8, 10, 250, out_permille=400),
        synth.make_cifar_resnet(22, "bf16", 2, 400, widths=(4, 8, 12), size=12, out_permille=300),
        synth.make_imagenet_basic_resnet(23, "bf16", (2, 1, 2, 1), 300, widths=(4, 8, 8, 12), size=32,
                                         classes=7, out_permille=500),
        synth.make_imagenet_bottleneck_resnet(24, "bf16", (2, 2, 1, 1), 500, widths=(4, 4, 8, 8),
                                              size=32, classes=5, out_permille=300),
    ]


@pytest.mark.parametrize("mi", range(4))
def test_only_identity_blocks_lose_output_filters(mi):
    model = stream_models()[mi]
    masks = orc.select_masks(model)
    seen = 0
    for bi, blk in enumerate(model["blocks"]):
        last = len(blk["convs"]) - 1
        if blk["shortcut"]["kind"] == "identity":
            m = masks[(bi, last)]
            k = blk["convs"][last]["W"].shape[0]
            assert int(m.sum()) == k - orc.prune_count(k, blk["prune_permille"][last]) < k
            seen += 1
        else:
            assert (bi, last) not in masks
    assert seen


def test_block_output_with_removed_filters_by_hand():
    """One block: the output channels whose filter went are relu(x) alone, the
    others are those of the block with all its output filters (their filters and
    what they read are untouched)."""
    model = synth.make_block_model(25, "bf16", 8, 9, 0, out_permille=500)
    x = np.abs(synth.make_input(95, 2, model["in_shape"]))
    masks = orc.select_masks(model)
    assert list(masks) == [(0, 1)]
    keep = masks[(0, 1)].astype(bool)
    assert keep.sum() == 4
    full = orc.forward(model, x)
    pruned = orc.forward(model, x, masks=masks)
    assert np.array_equal(pruned[:, keep], full[:, keep])
    assert np.array_equal(pruned[:, ~keep], np.maximum(x[:, ~keep].astype(np.float64), 0.0))
    assert not np.array_equal(pruned[:, ~keep], full[:, ~keep])
    ref = torch_forward(orc.zero_masked(model, masks), x)
    np.testing.assert_allclose(pruned, ref, rtol=1e-10, atol=1e-10 * np.abs(ref).max())


@pytest.mark.parametrize("mi", range(4))
def test_removed_output_filters_equal_zeroed_filters(mi):
    """The thin network, whose last convolution adds into the kept channels of the
    full-width block output, gives bit for bit the zero-masked network's result."""
    model = stream_models()[mi]
    x = synth.make_input(94, 2, model["in_shape"])
    masks = orc.select_masks(model)
    zeroed = orc.forward(model, x, masks=masks)
    thin = orc.extract(model, masks)
    n_stream = 0
    for (bi, ci), m in masks.items():
        blk = thin["blocks"][bi]
        assert blk["convs"][ci]["W"].shape[0] == int(m.sum())
        if ci + 1 == len(blk["convs"]):
            assert np.array_equal(blk["stream_keep"], np.flatnonzero(m))
            n_stream += 1
    assert n_stream
    assert np.array_equal(zeroed, orc.forward(thin, x))
    ref = torch_forward(orc.zero_masked(model, masks), x)
    np.testing.assert_allclose(zeroed, ref, rtol=1e-10, atol=1e-10 * np.abs(ref).max())
    inner = {k: v for k, v in masks.items() if k[1] + 1 < len(model["blocks"][k[0]]["convs"])}
    assert not np.array_equal(zeroed, orc.forward(model, x, masks=inner))


def test_output_filters_beside_a_projection_cannot_be_removed():
    model = synth.make_imagenet_basic_resnet(26, "bf16", (1, 1), 300, widths=(4, 8), size=16, classes=3)
    blk = model["blocks"][1]
    assert blk["shortcut"]["kind"] == "projection"
    mask = np.ones(8, dtype=np.uint8)
    mask[0] = 0
    with pytest.raises(ValueError):
        orc.extract(model, {(1, 1): mask})


def test_trace_records_every_conv_site():
    model = small_models()[3]
    x = synth.make_input(95, 1, model["in_shape"])
    tr = []
    y = orc.forward(model, x, trace=tr)
    n_convs = 1 + sum(len(b["convs"]) + (b["shortcut"]["kind"] == "projection")
                      for b in model["blocks"]) + 1
    assert len(tr) == n_convs
    assert np.array_equal(tr[-1]["y"], y)


# ---- generator vs Table II -------------------------------------------------

def test_generators_follow_table2():
    path = os.path.join(os.path.dirname(__file__), "golden", "table2_architectures.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for name, stem, *stages, fcn in rows:
        rs, k0 = stem.split(",")
        r = int(rs.split("x")[0])
        widths = tuple(int(s.split("x")[0]) for s in stages)
        nblocks = tuple(int(s.split("x")[1]) for s in stages)
        if r == 3:
            assert len(set(nblocks)) == 1
            m = synth.make_cifar_resnet(1, "bf16", nblocks[0], 0, widths=widths)
        else:
            m = synth.make_imagenet_basic_resnet(1, "bf16", nblocks, 0, widths=widths, size=32)
        assert m["stem"]["conv"]["W"].shape[0] == int(k0)
        assert m["stem"]["conv"]["W"].shape[2:] == (r, r)
        got = [(b["convs"][0]["W"].shape[0], b["convs"][1]["W"].shape[0]) for b in m["blocks"]]
        want = [(w, w) for w, nb in zip(widths, nblocks) for _ in range(nb)]
        assert got == want
        assert all(c["W"].shape[2:] == (3, 3) for b in m["blocks"] for c in b["convs"])
        assert m["head"]["fc_W"].shape[0] == int(fcn)
        depth = 2 + sum(2 * nb for nb in nblocks)
        assert name == f"resnet{depth}"


def test_baseline_config_channel_counts():
    want = {1: {16: 10, 32: 20, 64: 39}, 2: {64: 45, 128: 90, 256: 180, 512: 359},
            3: {64: 32, 128: 64, 256: 128, 512: 256}}
    for idx, table in want.items():
        model, _ = synth.make_config(idx)
        for bi, ci, pm in synth.prunable_convs(model):
            n = model["blocks"][bi]["convs"][ci]["W"].shape[0]
            assert n - orc.prune_count(n, pm) == table[n]


# ---- aggressive operator fusion (Sec. IV-B) -------------------------------------------

def fusible_models():
    """Basic blocks with each kind of shortcut: identity, subsample + zero-pad,
    1 x 1 projection."""
    return [
        synth.make_cifar_resnet(21, "bf16", 2, 400, widths=(4, 8, 12), size=12, classes=5),
        synth.make_imagenet_basic_resnet(22, "bf16", (1, 2, 1, 1), 300, widths=(4, 8, 8, 12), size=32,
                                         classes=7),
    ]


@pytest.mark.parametrize("mi", range(2))
def test_aggressive_fusion_is_an_equivalence(mi):
    """The fused model - auxiliary and padded convolutions concatenated, batch
    norms adjusted, no addition - computes what the original computes
    (Sec. IV-B: "the output of the neural network remains unchanged").  The
    original is evaluated by the walker pinned above; a wrong inverse of the
    batch norm on the filter-wise auxiliary weights, a misplaced identity tap or
    a lost projection shift all break this."""
    model = fusible_models()[mi]
    x = synth.make_input(97, 2, model["in_shape"])
    fused = orc.aggressive_fuse(model)
    a = orc.forward(model, x)
    b = orc.forward(fused, x)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-10 * np.abs(a).max())
    for blk in fused["blocks"]:
        assert blk["shortcut"]["kind"] == "none"


@pytest.mark.parametrize("mi,stages", [(0, 0), (0, 1), (0, 2), (1, 1), (1, 2), (1, 3)])
def test_fusion_option_x_of_n_is_an_equivalence(mi, stages):
    """The fusion option x/n (Sec. V, optimization setting): the blocks of the
    first x stages are fused, the others keep their addition; whichever x, the
    network computes what the original computes, and exactly the blocks of
    those stages lose their addition."""
    model = fusible_models()[mi]
    x = synth.make_input(98, 2, model["in_shape"])
    part = orc.aggressive_fuse(model, stages=stages)
    a = orc.forward(model, x)
    b = orc.forward(part, x)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-10 * np.abs(a).max())
    for blk_o, blk_f in zip(model["blocks"], part["blocks"]):
        fused = blk_f["shortcut"]["kind"] == "none"
        assert fused == (blk_o["stage"] < stages)
        if not fused:
            assert blk_f is blk_o
    n_stages = 1 + max(b["stage"] for b in model["blocks"])
    whole = orc.aggressive_fuse(model, stages=n_stages)
    assert all(b["shortcut"]["kind"] == "none" for b in whole["blocks"])
    # pruning the partially fused model: fused operators lose n - m, the others p * n (Alg. 1)
    masks = orc.select_masks(part)
    for bi, blk in enumerate(part["blocks"]):
        n = blk["convs"][0]["W"].shape[0]
        lost = int((masks[(bi, 0)] == 0).sum()) if (bi, 0) in masks else 0
        if blk["shortcut"]["kind"] == "none":
            assert lost == n - blk["original_filters"][0]
        else:
            assert lost == orc.prune_count(n, blk["prune_permille"][0])


def test_aggressive_fusion_shapes_and_auxiliary_values():
    """conv1' is (k + c) x c x 3 x 3 and conv2' is k x (k + c) x 3 x 3
    (Sec. IV-B-1); the channel-wise auxiliary filters are identities with an
    auxiliary batch norm omega = 1, lambda = 0; the filter-wise auxiliary weights
    are the inverse of the batch norm after conv2 (Sec. IV-B-2)."""
    model = fusible_models()[0]
    blk = model["blocks"][0]                      # identity shortcut
    k, c = blk["convs"][0]["W"].shape[:2]
    f = orc.aggressive_fuse_block(blk)
    w1, w2 = f["convs"][0]["W"], f["convs"][1]["W"]
    assert w1.shape == (k + c, c, 3, 3) and w2.shape == (k, k + c, 3, 3)
    assert np.array_equal(w1[:k], blk["convs"][0]["W"]) and np.array_equal(w2[:, :k], blk["convs"][1]["W"])
    assert np.array_equal(w1[k:], identity_weights(c))
    bn1 = f["bns"][0]
    omega_aux = bn1["gamma"][k:] / np.sqrt(bn1["var"][k:] + bn1["eps"])
    assert np.array_equal(omega_aux, np.ones(c))
    assert not bn1["beta"][k:].any() and not bn1["mean"][k:].any()
    b2 = blk["bns"][1]
    omega2 = b2["gamma"].astype(np.float64) / np.sqrt(b2["var"].astype(np.float64) + b2["eps"])
    aux = w2[:, k:]
    assert np.allclose(aux[np.arange(k), np.arange(k), 1, 1] * omega2, 1.0, rtol=1e-15)
    assert np.count_nonzero(aux) == k
    assert f["original_filters"] == [k, k]


def test_fused_operator_loses_n_minus_m_filters():
    """Alg. 1: a fused operator with n filters, m of them original, loses its
    n - m lowest-norm filters; conv2' (n = m) loses none."""
    model = fusible_models()[1]
    fused = orc.aggressive_fuse(model)
    masks = orc.select_masks(fused)
    for bi, blk in enumerate(fused["blocks"]):
        n, c = blk["convs"][0]["W"].shape[:2]
        m = blk["original_filters"][0]
        assert n - m == c
        assert int((masks[(bi, 0)] == 0).sum()) == n - m
        assert (bi, 1) not in masks
    # the thinner model equals the fused model with those filters zeroed
    x = synth.make_input(96, 2, model["in_shape"])
    a = orc.forward(fused, x, masks=masks)
    b = orc.forward(orc.extract(fused, masks), x)
    assert np.array_equal(a, b)


def test_fusion_needs_an_invertible_batch_norm():
    blk = dict(fusible_models()[0]["blocks"][0])
    blk["bns"] = [dict(b) for b in blk["bns"]]
    g = blk["bns"][1]["gamma"].copy()
    g[2] = 0.0
    blk["bns"][1]["gamma"] = g
    with pytest.raises(ZeroDivisionError):
        orc.aggressive_fuse_block(blk)
