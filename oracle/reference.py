"""Plain evaluation of a residual network as the paper states it, on the CPU.

TEST INFRASTRUCTURE ONLY: the GPU library never imports this module.

The network is evaluated operator by operator in its ORIGINAL form -
convolution, then batch normalisation in its literal (gamma, beta, mean, var,
eps) form, then ReLU, and an element-wise addition at the end of every
building block (Sec. III; Table II) - in double precision on NCHW tensors,
through the C routines of fupr_oracle.c.  Pruned filters are "masked by zero
matrices" (Sec. IV-C): the network keeps its full width and the masked
filters, together with their batch-norm scale and shift, are set to zero.

Two further evaluators exist only so that tests can pin this one against the
paper's equivalence claims:
  * fold()/forward(..., merged=True): batch norm written as omega*x + lambda
    (Eq. 3-5) and merged into the preceding convolution (Sec. VI-B-3);
  * extract(): the thinner model obtained when masked filters are removed
    (last step of Alg. 1).

aggressive_fuse() builds the "dilated" model of Sec. IV-B (auxiliary and padded
convolutions concatenated to a basic block's two convolutions, batch norms
adjusted, the element-wise addition gone); the same walker evaluates it.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfupr_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().orc_num_threads())


def _p(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_D)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# --------------------------------------------------------------------------
# operators
# --------------------------------------------------------------------------

def conv2d(x, w, stride, pad):
    """Convolution operator k x c x r x s (Sec. IV-B-1 notation), zero padding."""
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2
    p = (h + 2 * pad - r) // stride + 1
    q = (wd + 2 * pad - s) // stride + 1
    y = np.empty((n, k, p, q), dtype=np.float64)
    _load().orc_conv2d(_p(x), _p(w), _p(y), n, c, h, wd, k, r, s, stride, pad)
    return y


def batchnorm(x, bn):
    """gamma * (x - mean) / sqrt(var + eps) + beta (Sec. IV-B-2)."""
    x = _f64(x)
    n, k, h, w = x.shape
    y = np.empty_like(x)
    _load().orc_batchnorm(_p(x), _p(y), _p(_f64(bn["gamma"])), _p(_f64(bn["beta"])),
                          _p(_f64(bn["mean"])), _p(_f64(bn["var"])),
                          ctypes.c_double(float(bn["eps"])), n, k, h * w)
    return y


def relu(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().orc_relu(_p(x), _p(y), ctypes.c_size_t(x.size))
    return y


def add(a, b):
    a, b = _f64(a), _f64(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    _load().orc_add(_p(a), _p(b), _p(y), ctypes.c_size_t(a.size))
    return y


def shortcut_subsample_pad(x, k, stride):
    """Parameter-free shortcut: x[:, :, ::stride, ::stride], zero channels up to k."""
    x = _f64(x)
    n, c, h, w = x.shape
    p, q = (h + stride - 1) // stride, (w + stride - 1) // stride
    y = np.empty((n, k, p, q), dtype=np.float64)
    _load().orc_shortcut_subsample_pad(_p(x), _p(y), n, c, h, w, k, stride)
    return y


def maxpool(x, k, stride, pad):
    x = _f64(x)
    n, c, h, w = x.shape
    p = (h + 2 * pad - k) // stride + 1
    q = (w + 2 * pad - k) // stride + 1
    y = np.empty((n, c, p, q), dtype=np.float64)
    _load().orc_maxpool(_p(x), _p(y), n, c, h, w, k, stride, pad)
    return y


def global_mean(x):
    x = _f64(x)
    n, c, h, w = x.shape
    y = np.empty((n, c), dtype=np.float64)
    _load().orc_global_mean(_p(x), _p(y), n, c, h * w)
    return y


def fc(x, w, b):
    x, w, b = _f64(x), _f64(w), _f64(b)
    n, i = x.shape
    o = w.shape[0]
    y = np.empty((n, o), dtype=np.float64)
    _load().orc_fc(_p(x), _p(w), _p(b), _p(y), n, i, o)
    return y


# --------------------------------------------------------------------------
# filter selection (Sec. IV-C, Eq. 6 and Alg. 1)
# --------------------------------------------------------------------------

def filter_norms(w, norm=2):
    """l1 or l2 norm of every filter W_k over (c, r, s), sequential double sum."""
    w = _f64(w)
    k = w.shape[0]
    out = np.empty(k, dtype=np.float64)
    _load().orc_filter_norms(_p(w), k, w.size // k, int(norm), _p(out))
    return out


def prune_count(n, permille):
    """Number of filters a non-fused operator loses: floor(p_phi * n), in integers,
    never all of them."""
    return min((n * int(permille)) // 1000, n - 1)


def select_mask(w, n_prune, norm=1):
    """mask[k] = 0 for the n_prune filters of lowest norm (ties: lower index
    first), 1 for the filters that stay."""
    norms = filter_norms(w, norm)
    order = np.argsort(norms, kind="stable")
    mask = np.ones(w.shape[0], dtype=np.uint8)
    mask[order[:n_prune]] = 0
    return mask


def select_masks(model, norm=1):
    """{(block, conv): mask} for every conv that loses filters; norms are taken
    on the raw (unfolded) weights.  A fused operator with n filters, m of them
    original, loses the n - m of lowest norm; any other operator with a nonzero
    rate loses floor(p_phi n) (Alg. 1)."""
    masks = {}
    for bi, blk in enumerate(model["blocks"]):
        original = blk.get("original_filters")
        for ci, pm in enumerate(blk["prune_permille"]):
            w = blk["convs"][ci]["W"]
            if original is not None:
                n_prune = w.shape[0] - original[ci]
            else:
                n_prune = prune_count(w.shape[0], pm) if pm else 0
            if n_prune:
                masks[(bi, ci)] = select_mask(w, n_prune, norm)
    return masks


def zero_masked(model, masks):
    """The same network with every masked filter, and that channel's batch-norm
    scale and shift, set to zero.  Widths do not change."""
    out = dict(model)
    out["blocks"] = []
    for bi, blk in enumerate(model["blocks"]):
        nb = dict(blk)
        nb["convs"] = [dict(c) for c in blk["convs"]]
        nb["bns"] = [dict(b) for b in blk["bns"]]
        for ci in range(len(blk["convs"])):
            m = masks.get((bi, ci))
            if m is None:
                continue
            keep = m.astype(bool)
            w = nb["convs"][ci]["W"].copy()
            w[~keep] = 0
            nb["convs"][ci]["W"] = w
            for key in ("gamma", "beta"):
                v = nb["bns"][ci][key].copy()
                v[~keep] = 0
                nb["bns"][ci][key] = v
        out["blocks"].append(nb)
    return out


def extract(model, masks):
    """The thinner network left when masked filters are removed: the producer
    loses those filters (and batch-norm channels), the next conv of the block
    loses the matching input channels.  A block's LAST conv has no next conv:
    its kept filters are recorded as the block's "stream_keep", the channels of
    the block's full-width output they add to (identity shortcut only; the other
    channels of the output are the shortcut's alone)."""
    out = dict(model)
    out["blocks"] = []
    for bi, blk in enumerate(model["blocks"]):
        nb = dict(blk)
        nb["convs"] = [dict(c) for c in blk["convs"]]
        nb["bns"] = [dict(b) for b in blk["bns"]]
        nb["prune_permille"] = [0] * len(blk["convs"])
        for ci in range(len(blk["convs"])):
            m = masks.get((bi, ci))
            if m is None:
                continue
            keep = np.flatnonzero(m)
            nb["convs"][ci]["W"] = np.ascontiguousarray(nb["convs"][ci]["W"][keep])
            for key in ("gamma", "beta", "mean", "var"):
                nb["bns"][ci][key] = np.ascontiguousarray(nb["bns"][ci][key][keep])
            if ci + 1 < len(blk["convs"]):
                nxt = nb["convs"][ci + 1]
                nxt["W"] = np.ascontiguousarray(nxt["W"][:, keep])
            else:
                if blk["shortcut"]["kind"] != "identity":
                    raise ValueError("output filters are removed only beside an identity shortcut")
                nb["stream_keep"] = keep
        out["blocks"].append(nb)
    return out


# --------------------------------------------------------------------------
# batch norm as an affine map, merged into the convolution before it
# --------------------------------------------------------------------------

def fold(w, bn, conv_bias=None):
    """omega = gamma / sqrt(var + eps), lambda = beta - omega * mean (Eq. 3-5);
    W'_k = omega_k W_k, b'_k = lambda_k + omega_k b_k."""
    w = _f64(w)
    omega = _f64(bn["gamma"]) / np.sqrt(_f64(bn["var"]) + float(bn["eps"]))
    lam = _f64(bn["beta"]) - omega * _f64(bn["mean"])
    wf = w * omega[:, None, None, None]
    bf = lam if conv_bias is None else lam + omega * _f64(conv_bias)
    return wf, bf


def _conv_bn(x, conv, bn, merged):
    if merged:
        wf, bf = fold(conv["W"], bn)
        return conv2d(x, wf, conv["stride"], conv["pad"]) + bf[None, :, None, None]
    return batchnorm(conv2d(x, conv["W"], conv["stride"], conv["pad"]), bn)


# --------------------------------------------------------------------------
# aggressive operator fusion (Sec. IV-B)
# --------------------------------------------------------------------------

def _omega_lambda(bn):
    omega = _f64(bn["gamma"]) / np.sqrt(_f64(bn["var"]) + float(bn["eps"]))
    return omega, _f64(bn["beta"]) - omega * _f64(bn["mean"])


def aggressive_fuse_block(blk):
    """A basic residual block (two r x s convolutions, a shortcut, an addition)
    rewritten as two dilated convolutions and no addition (Sec. IV-B-1, the
    basic-block and projection-shortcut recipes; batch norms per Sec. IV-B-2).

    With conv1 = k1 x c x r x s, conv2 = k2 x k1 x r x s:
      * an auxiliary convolution for channel-wise fusion, identity weights (a 1
        at the centre tap of filter j, channel j), is concatenated to conv1
        along the filters: (k1 + c) x c x r x s; its c outputs are the block
        input (at conv1's stride).  An auxiliary batch norm with omega = 1,
        lambda = 0 goes with them.
      * an auxiliary convolution for filter-wise fusion is concatenated to conv2
        along the channels: k2 x (k1 + c) x r x s, reading the copied input.
        The batch norm after conv2 stays and would scale what the auxiliary
        weights add, so they hold its inverse: 1 / omega2_k at (k, k, centre)
        for an identity (or subsample-and-zero-pad) shortcut.  A 1 x 1
        projection on the shortcut becomes a padded r x s convolution whose
        centre tap is omega_p,k / omega2_k * Wp[k, :]; its shift lambda_p goes
        into the shift of the batch norm after conv2.

    The copy of the input passes through the block's first ReLU, so the rewrite
    is exact for block inputs that are outputs of a ReLU (every block of the
    Table II networks).  Returns the fused block; "original_filters" records m
    of Alg. 1 for both operators.
    """
    if blk["kind"] != "basic":
        raise ValueError("only basic blocks are fused")
    c1, c2 = blk["convs"]
    b1, b2 = blk["bns"]
    w1, w2 = _f64(c1["W"]), _f64(c2["W"])
    k1, c, r, s_ = w1.shape
    k2 = w2.shape[0]
    assert w2.shape[1:] == (k1, r, s_) and r % 2 == 1 and s_ % 2 == 1
    assert c1["pad"] == r // 2 and c2["pad"] == r // 2 and c2["stride"] == 1
    cr, cs = r // 2, s_ // 2
    sc = blk["shortcut"]

    aux_c = np.zeros((c, c, r, s_))
    aux_c[np.arange(c), np.arange(c), cr, cs] = 1.0
    w1f = np.concatenate([w1, aux_c], axis=0)
    eps1 = float(b1["eps"])
    bn1f = {"gamma": np.concatenate([_f64(b1["gamma"]), np.full(c, np.sqrt(1.0 + eps1))]),
            "beta": np.concatenate([_f64(b1["beta"]), np.zeros(c)]),
            "mean": np.concatenate([_f64(b1["mean"]), np.zeros(c)]),
            "var": np.concatenate([_f64(b1["var"]), np.ones(c)]),
            "eps": eps1}

    omega2, _ = _omega_lambda(b2)
    if np.any(omega2 == 0.0):
        raise ZeroDivisionError("the batch norm after conv2 has a zero scale")
    aux_f = np.zeros((k2, c, r, s_))
    beta2 = _f64(b2["beta"]).copy()
    if sc["kind"] in ("identity", "optionA"):
        assert c <= k2 and (sc["kind"] == "optionA" or c == k2)
        assert c1["stride"] == (sc["stride"] if sc["kind"] == "optionA" else 1)
        aux_f[np.arange(c), np.arange(c), cr, cs] = 1.0 / omega2[:c]
    elif sc["kind"] == "projection":
        wp = _f64(sc["conv"]["W"])
        assert wp.shape == (k2, c, 1, 1) and sc["conv"]["pad"] == 0
        assert sc["conv"]["stride"] == c1["stride"]
        omega_p, lambda_p = _omega_lambda(sc["bn"])
        aux_f[:, :, cr, cs] = (omega_p / omega2)[:, None] * wp[:, :, 0, 0]
        beta2 += lambda_p
    else:
        raise ValueError(sc["kind"])
    w2f = np.concatenate([w2, aux_f], axis=1)
    bn2f = dict(b2)
    bn2f["beta"] = beta2

    return {"kind": "basic",
            "convs": [{"W": w1f, "stride": c1["stride"], "pad": c1["pad"]},
                      {"W": w2f, "stride": 1, "pad": c2["pad"]}],
            "bns": [bn1f, bn2f],
            "prune_permille": [0, 0],
            "original_filters": [k1, k2],
            "shortcut": {"kind": "none"}}


def aggressive_fuse(model, stages=None):
    """The model with its basic blocks rewritten by aggressive_fuse_block.

    stages: the fusion option x of "x/n" (Sec. V, optimization setting): only the
    blocks of the first x stages are fused, in order; None fuses every stage."""
    out = dict(model)
    out["blocks"] = [aggressive_fuse_block(b)
                     if b["kind"] == "basic" and (stages is None or b.get("stage", 0) < stages) else b
                     for b in model["blocks"]]
    return out


# --------------------------------------------------------------------------
# network
# --------------------------------------------------------------------------

def forward(model, x, masks=None, merged=False, trace=None):
    """Output of the network for images x (N, C, H, W).

    masks: {(block, conv): mask}; masked filters are zeroed (see zero_masked).
    merged: evaluate conv+bn through the merged form (for equivalence tests).
    trace: if a list, one record per convolution site is appended:
        {"site", "x", "res", "y"} with the conv's input, the tensor added
        before the final ReLU (or None) and the site's output (after bn, add
        and ReLU as the site has them).
    Returns logits (N, classes) if the model has a head, else the last block's
    output (N, K, P, Q).
    """
    if masks:
        model = zero_masked(model, masks)
    x = _f64(x)

    def rec(site, xin, res, y):
        if trace is not None:
            trace.append({"site": site, "x": xin, "res": res, "y": y})

    stem = model["stem"]
    if stem is not None:
        y = relu(_conv_bn(x, stem["conv"], stem["bn"], merged))
        rec("stem", x, None, y)
        x = y
        if stem["maxpool"] is not None:
            k, st, pd = stem["maxpool"]
            x = maxpool(x, k, st, pd)
    for bi, blk in enumerate(model["blocks"]):
        convs, bns = blk["convs"], blk["bns"]
        sc = blk["shortcut"]
        k_out = convs[-1]["W"].shape[0]
        if sc["kind"] == "none":
            short = None
        elif sc["kind"] == "identity":
            short = x
        elif sc["kind"] == "optionA":
            short = shortcut_subsample_pad(x, k_out, sc["stride"])
        else:
            short = _conv_bn(x, sc["conv"], sc["bn"], merged)
            rec(f"b{bi}.proj", x, None, short)
        h = x
        for ci in range(len(convs) - 1):
            y = relu(_conv_bn(h, convs[ci], bns[ci], merged))
            rec(f"b{bi}.conv{ci + 1}", h, None, y)
            h = y
        y = _conv_bn(h, convs[-1], bns[-1], merged)
        keep = blk.get("stream_keep")
        if keep is not None:
            # removed output filters contribute nothing: the kept ones go to their
            # own channels of a full-width tensor of zeros
            wide = np.zeros_like(short)
            wide[:, keep] = y
            y = wide
        y = relu(y if short is None else add(y, short))
        rec(f"b{bi}.conv{len(convs)}", h, short, y)
        x = y
    head = model["head"]
    if head is None:
        return x
    pooled = global_mean(x)
    logits = fc(pooled, head["fc_W"], head["fc_b"])
    rec("fc", pooled, None, logits)
    return logits
