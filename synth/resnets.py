"""Seeded descriptions of the residual networks used as workloads.

A *model* is plain data describing the original (unfused, unpruned) network in
the notation of the paper: convolution operators with weights k x c x r x s
(Sec. IV-B-1), batch-normalisation operators given by (gamma, beta, mean, var,
eps) (Sec. IV-B-2, Eq. 3-5), building blocks that end in an element-wise
addition (Table II), and a per-convolution pruning rate p_phi in permille
(Alg. 1).  Nothing here evaluates the network.

Layout of a model (all arrays numpy float32, C-contiguous):

    model = {
      "name": str, "dtype": "f32" | "bf16" | "f16",
      "in_shape": (C, H, W),
      "stem": None | {"conv": conv, "bn": bn, "maxpool": None | (k, stride, pad)},
      "blocks": [block, ...],
      "head": None | {"fc_W": (out, in), "fc_b": (out,)},  # global mean + fc
    }
    conv  = {"W": (K, C, R, S), "stride": int, "pad": int}
    bn    = {"gamma", "beta", "mean", "var": (K,), "eps": float}
    block = {"kind": "basic" | "bottleneck",
             "stage": int,                   # which stage of Table II the block belongs to
             "convs": [conv, ...], "bns": [bn, ...],
             "prune_permille": [int, ...],   # one per conv, 0 = not pruned; a nonzero
                                             # rate on the LAST conv prunes the block's
                                             # output filters (identity shortcut only)
             "shortcut": {"kind": "identity"}
                       | {"kind": "optionA", "stride": 2}
                       | {"kind": "projection", "conv": conv, "bn": bn}}

Value distributions (the same for every workload): images and block inputs
x ~ N(0, 1); conv weights He-normal on the unpruned shape, W ~ N(0, 2/(c r s));
gamma ~ U(0.5, 1.5); beta ~ N(0, 0.1^2); mean ~ N(0, 0.1^2); var ~ U(0.5, 1.5);
eps = 1e-5; fc weights ~ N(0, 1/fan_in), fc bias 0.

Random streams: numpy default_rng([BASE_SEED + config_index, stream]) with
stream 0 = images, 1 = parameters (drawn in graph order; per conv: W, then its
bn's gamma, beta, mean, var; shortcut conv after the block's own convs; fc
last), 2 = per-layer pruning rates (config 4 only).
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 201016165

CONFIG_NAMES = [
    "cifar-basic-block-f32",
    "resnet56-cifar-bf16",
    "resnet18-imagenet-bf16",
    "resnet50-imagenet-bf16",
    "resnet50-imagenet-f16-irregular",
]

_EPS = 1e-5


def _conv(rng, k, c, r, s, stride, pad):
    std = np.sqrt(2.0 / (c * r * s))
    w = rng.standard_normal((k, c, r, s), dtype=np.float64) * std
    return {"W": np.ascontiguousarray(w, dtype=np.float32), "stride": int(stride), "pad": int(pad)}


def _bn(rng, k):
    gamma = rng.uniform(0.5, 1.5, k)
    beta = rng.standard_normal(k) * 0.1
    mean = rng.standard_normal(k) * 0.1
    var = rng.uniform(0.5, 1.5, k)
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    return {"gamma": f(gamma), "beta": f(beta), "mean": f(mean), "var": f(var), "eps": _EPS}


def _conv_bn(rng, k, c, r, s, stride, pad):
    cv = _conv(rng, k, c, r, s, stride, pad)
    return cv, _bn(rng, k)


def _basic_block(rng, c_in, k, stride, shortcut, permille, out_permille=0):
    c1, b1 = _conv_bn(rng, k, c_in, 3, 3, stride, 1)
    c2, b2 = _conv_bn(rng, k, k, 3, 3, 1, 1)
    blk = {"kind": "basic", "convs": [c1, c2], "bns": [b1, b2],
           "prune_permille": [int(permille), int(out_permille) if shortcut == "identity" else 0]}
    if shortcut == "projection":
        sc, sb = _conv_bn(rng, k, c_in, 1, 1, stride, 0)
        blk["shortcut"] = {"kind": "projection", "conv": sc, "bn": sb}
    elif shortcut == "optionA":
        blk["shortcut"] = {"kind": "optionA", "stride": int(stride)}
    else:
        blk["shortcut"] = {"kind": "identity"}
    return blk


def _bottleneck_block(rng, c_in, width, stride, projection, permilles, out_permille=0):
    k_out = 4 * width
    c1, b1 = _conv_bn(rng, width, c_in, 1, 1, 1, 0)
    c2, b2 = _conv_bn(rng, width, width, 3, 3, stride, 1)
    c3, b3 = _conv_bn(rng, k_out, width, 1, 1, 1, 0)
    blk = {"kind": "bottleneck", "convs": [c1, c2, c3], "bns": [b1, b2, b3],
           "prune_permille": [int(permilles[0]), int(permilles[1]),
                              0 if projection else int(out_permille)]}
    if projection:
        sc, sb = _conv_bn(rng, k_out, c_in, 1, 1, stride, 0)
        blk["shortcut"] = {"kind": "projection", "conv": sc, "bn": sb}
    else:
        blk["shortcut"] = {"kind": "identity"}
    return blk


def _head(rng, n_in, n_out):
    w = rng.standard_normal((n_out, n_in)) * np.sqrt(1.0 / n_in)
    return {"fc_W": np.ascontiguousarray(w, dtype=np.float32),
            "fc_b": np.zeros(n_out, dtype=np.float32)}


def make_block_model(seed, dtype="f32", channels=16, size=32, permille=250, out_permille=0):
    """One CIFAR-style basic block with identity shortcut (config 0)."""
    rng = np.random.default_rng([seed, 1])
    blk = _basic_block(rng, channels, channels, 1, "identity", permille, out_permille)
    blk["stage"] = 0
    return {"name": "basic-block", "dtype": dtype, "in_shape": (channels, size, size),
            "stem": None, "blocks": [blk], "head": None}


def make_cifar_resnet(seed, dtype="bf16", blocks_per_stage=9, permille=400,
                      widths=(16, 32, 64), size=32, classes=10, out_permille=0):
    """CIFAR residual network of Table II (3x3/16 stem, three stages, fc 10)
    with option-A shortcuts where the resolution halves."""
    rng = np.random.default_rng([seed, 1])
    sc, sb = _conv_bn(rng, widths[0], 3, 3, 3, 1, 1)
    blocks = []
    c_in = widths[0]
    for si, k in enumerate(widths):
        for bi in range(blocks_per_stage):
            down = si > 0 and bi == 0
            blocks.append(_basic_block(rng, c_in, k, 2 if down else 1,
                                       "optionA" if down else "identity", permille,
                                       out_permille))
            blocks[-1]["stage"] = si
            c_in = k
    return {"name": f"cifar-resnet{6 * blocks_per_stage + 2}", "dtype": dtype,
            "in_shape": (3, size, size),
            "stem": {"conv": sc, "bn": sb, "maxpool": None},
            "blocks": blocks, "head": _head(rng, c_in, classes)}


def make_imagenet_basic_resnet(seed, dtype="bf16", stage_blocks=(2, 2, 2, 2), permille=300,
                               widths=(64, 128, 256, 512), size=224, classes=1000,
                               out_permille=0):
    """ImageNet residual network of Table II (7x7/64 stem, max-pool, four
    stages of basic blocks, fc 1000) with projection shortcuts."""
    rng = np.random.default_rng([seed, 1])
    sc, sb = _conv_bn(rng, widths[0], 3, 7, 7, 2, 3)
    blocks = []
    c_in = widths[0]
    for si, k in enumerate(widths):
        for bi in range(stage_blocks[si]):
            down = si > 0 and bi == 0
            blocks.append(_basic_block(rng, c_in, k, 2 if down else 1,
                                       "projection" if down else "identity", permille,
                                       out_permille))
            blocks[-1]["stage"] = si
            c_in = k
    return {"name": f"imagenet-resnet{2 * sum(stage_blocks) + 2}", "dtype": dtype,
            "in_shape": (3, size, size),
            "stem": {"conv": sc, "bn": sb, "maxpool": (3, 2, 1)},
            "blocks": blocks, "head": _head(rng, c_in, classes)}


def make_imagenet_bottleneck_resnet(seed, dtype="bf16", stage_blocks=(3, 4, 6, 3),
                                    permille=500, permille_range=None,
                                    widths=(64, 128, 256, 512), size=224, classes=1000,
                                    out_permille=0):
    """Bottleneck residual network (1x1, 3x3, 1x1 with 4x expansion; stride on
    the 3x3).  permille_range=(lo, hi) draws one rate per prunable conv."""
    rng = np.random.default_rng([seed, 1])
    prng = np.random.default_rng([seed, 2])
    sc, sb = _conv_bn(rng, widths[0], 3, 7, 7, 2, 3)
    blocks = []
    c_in = widths[0]
    for si, w in enumerate(widths):
        for bi in range(stage_blocks[si]):
            stride = 2 if (si > 0 and bi == 0) else 1
            if permille_range is None:
                pm = (permille, permille)
            else:
                lo, hi = permille_range
                pm = tuple(int(np.floor(prng.uniform(lo, hi))) for _ in range(2))
            blocks.append(_bottleneck_block(rng, c_in, w, stride, bi == 0, pm, out_permille))
            blocks[-1]["stage"] = si
            c_in = 4 * w
    return {"name": f"imagenet-resnet{3 * sum(stage_blocks) + 2}", "dtype": dtype,
            "in_shape": (3, size, size),
            "stem": {"conv": sc, "bn": sb, "maxpool": (3, 2, 1)},
            "blocks": blocks, "head": _head(rng, c_in, classes)}


_DEFAULT_BATCH = [1, 128, 64, 64, 256]


def make_config(index):
    """Model and default batch size of benchmark configuration `index` (0..4)."""
    seed = BASE_SEED + index
    if index == 0:
        m = make_block_model(seed, "f32", 16, 32, 250)
    elif index == 1:
        m = make_cifar_resnet(seed, "bf16", 9, 400)
    elif index == 2:
        m = make_imagenet_basic_resnet(seed, "bf16", (2, 2, 2, 2), 300)
    elif index == 3:
        m = make_imagenet_bottleneck_resnet(seed, "bf16", (3, 4, 6, 3), 500)
    elif index == 4:
        m = make_imagenet_bottleneck_resnet(seed, "f16", (3, 4, 6, 3), permille_range=(100, 700))
    else:
        raise ValueError(f"no such config: {index}")
    m["config_index"] = index
    m["name"] = CONFIG_NAMES[index]
    return m, _DEFAULT_BATCH[index]


# The networks the paper itself measures (Table II; Tables V-VI are latencies at
# batch 1): seeds BASE_SEED + 10 + position in this list.
PAPER_WORKLOADS = ["resnet20", "resnet32", "resnet18", "resnet34"]


def make_paper_workload(name, permille=300, dtype="bf16", out_permille=0):
    """ResNet-20 / 32 on 32 x 32 images, ResNet-18 / 34 on 224 x 224 images, every
    block's first convolution pruned at `permille` (the paper's rates are 0, 100,
    200, 300).  out_permille: the rate of the last convolution of every block with
    an identity shortcut (the paper prunes all non-fused convolutions at one rate,
    Sec. V-A; the blocks whose shortcut changes shape keep their output filters)."""
    seed = BASE_SEED + 10 + PAPER_WORKLOADS.index(name)
    if name == "resnet20":
        m = make_cifar_resnet(seed, dtype, 3, permille, out_permille=out_permille)
    elif name == "resnet32":
        m = make_cifar_resnet(seed, dtype, 5, permille, out_permille=out_permille)
    elif name == "resnet18":
        m = make_imagenet_basic_resnet(seed, dtype, (2, 2, 2, 2), permille,
                                       out_permille=out_permille)
    else:
        m = make_imagenet_basic_resnet(seed, dtype, (3, 4, 6, 3), permille,
                                       out_permille=out_permille)
    m["name"] = f"{name}-{dtype}-p{permille}" + (f"-out{out_permille}" if out_permille else "")
    return m


def make_input(seed, batch, in_shape, first=0):
    """Images first..first+batch-1 of the stream, NCHW float32, x ~ N(0, 1).

    Image i is drawn from its own generator so that any subset of a batch can
    be produced without drawing the rest."""
    c, h, w = in_shape
    out = np.empty((batch, c, h, w), dtype=np.float32)
    for i in range(batch):
        rng = np.random.default_rng([seed, 0, first + i])
        out[i] = rng.standard_normal((c, h, w), dtype=np.float32)
    return out


def prunable_convs(model):
    """[(block_index, conv_index, permille)] of the convs with a nonzero rate."""
    out = []
    for bi, blk in enumerate(model["blocks"]):
        for ci, pm in enumerate(blk["prune_permille"]):
            if pm:
                out.append((bi, ci, pm))
    return out
