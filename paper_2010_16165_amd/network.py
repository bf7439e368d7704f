"""From a pre-trained model description to a runnable fupr model (Sec. IV-A:
model + fusion options + pruning rates -> optimised model).

Orchestration only: every number is produced by the library calls
(fupr_select_filters, fupr_fold, fupr_prune, fupr_xconv_fuse, fupr_proj_concat,
fupr_pack); this module decides which call sees which layer, wires the blocks
(which tensor is a shortcut, where a projection sits), lays the packed blobs
out in one buffer, and in one place moves numbers without computing any: the
removed output filters of a 1 x 1 last convolution go back in as zero rows
(exact copies of the kept rows, zeros elsewhere).  A C caller of
fupr_model_create does the same wiring itself from the operator descriptions.
The model description is the plain-data format of synth.resnets.
"""
from __future__ import annotations

import numpy as np

from . import binding as B


class Layer:
    """One convolution site of the optimised network (host side)."""

    def __init__(self, site, W, bias, stride, pad, relu, add=False, keep=None, cat_stride=0):
        self.site = site
        self.cat_stride = cat_stride   # > 0: the last convolution with the block's projection
                                       # shortcut concatenated; the block input is read at this stride
        self.keep = keep        # int32 channels of the block output the kept filters add into
        self.W = W              # folded, compacted, float32 K x C x R x S
        self.bias = bias        # float32 K
        self.stride = stride
        self.pad = pad
        self.relu = relu
        self.add = add
        self.shape = B.shape_of(W, stride, pad)


def _fold(conv, bn):
    sh = B.shape_of(conv["W"], conv["stride"], conv["pad"])
    return B.fupr_fold(sh, conv["W"], None, bn["gamma"], bn["beta"], bn["mean"], bn["var"],
                       bn["eps"], B.FUSE_BN)


_SHORTCUTS = {"identity": B.SHORTCUT_IDENTITY, "optionA": B.SHORTCUT_SUBSAMPLE_PAD,
              "projection": B.SHORTCUT_PROJECTION}


def _aggressive(blk):
    """A basic block after aggressive fusion (Sec. IV-B): two dilated convolutions,
    no addition.  A fused operator loses n - m filters (Alg. 1), m = its original
    filter count; that is recorded as an explicit count."""
    sc = blk["shortcut"]
    c1, b1, c2, b2 = B.fupr_xconv_fuse(blk["convs"][0], blk["bns"][0], blk["convs"][1], blk["bns"][1],
                                       _SHORTCUTS[sc["kind"]], sc.get("conv"), sc.get("bn"))
    k1 = blk["convs"][0]["W"].shape[0]
    return {"kind": "basic", "convs": [c1, c2], "bns": [b1, b2], "prune_permille": [0, 0],
            "prune_counts": [c1["W"].shape[0] - k1, 0], "shortcut": {"kind": "none"}}


def optimise(model, norm=1, aggressive=False, prune_fused=True, fuse_stages=None,
             concat_projection=True):
    """Masks from the raw weights, batch norm merged, masked filters removed.

    aggressive: basic blocks are first rewritten by aggressive fusion; with
    prune_fused their dilated first operator then loses its n - m lowest-norm
    filters (Alg. 1), without it the fused model is run as it is.
    fuse_stages: the fusion option x of "x/n" (Sec. V, optimization setting): only
    the blocks of the first x stages are fused; None fuses every stage.
    concat_projection: a bottleneck block's projection shortcut is concatenated to
    its last 1 x 1 convolution (fupr_proj_concat, Sec. IV-B-1) and accumulates in
    that convolution's accumulators instead of running as an operator of its own
    (16-bit types).

    Returns {"layers": [Layer...], "masks": {(block, conv): uint8 mask},
             "keep_idx": {(block, conv): int32 indices}, "wiring": [...]}
    where wiring lists, per operator, what build() needs."""
    layers, masks, keeps, wiring = [], {}, {}, []
    stem = model["stem"]
    if stem is not None:
        Wf, bf = _fold(stem["conv"], stem["bn"])
        layers.append(Layer("stem", Wf, bf, stem["conv"]["stride"], stem["conv"]["pad"], True))
        wiring.append(("conv", len(layers) - 1, None))
        if stem["maxpool"] is not None:
            wiring.append(("maxpool", stem["maxpool"], None))
    for bi, blk in enumerate(model["blocks"]):
        if aggressive and blk["kind"] == "basic" and (fuse_stages is None
                                                      or blk.get("stage", 0) < fuse_stages):
            blk = _aggressive(blk)
            if not prune_fused:
                blk["prune_counts"] = [0, 0]
        convs, bns = blk["convs"], blk["bns"]
        folded = [list(_fold(c, b)) for c, b in zip(convs, bns)]
        counts = blk.get("prune_counts")
        for ci, pm in enumerate(blk["prune_permille"]):
            if not pm and not (counts and counts[ci]):
                continue
            raw = convs[ci]["W"]
            sh_raw = B.shape_of(raw, convs[ci]["stride"], convs[ci]["pad"])
            n_prune = counts[ci] if counts else B.fupr_prune_count(sh_raw.K, pm)
            mask = B.fupr_select_filters(sh_raw, raw, norm, n_prune)
            Wp, bp = folded[ci]
            prod = B.shape_of(Wp, convs[ci]["stride"], convs[ci]["pad"])
            if ci + 1 < len(convs):
                Wn = folded[ci + 1][0]
                cons = B.shape_of(Wn, convs[ci + 1]["stride"], convs[ci + 1]["pad"])
                keep, Wp_c, bp_c, (Wn_c,) = B.fupr_prune(prod, Wp, bp, mask, [cons], [Wn])
                folded[ci + 1][0] = Wn_c
            else:
                # the block's output filters: nothing downstream shrinks, the kept filters
                # add into their channels of the full-width output
                if blk["shortcut"]["kind"] != "identity":
                    raise ValueError("output filters are pruned only beside an identity shortcut")
                keep, Wp_c, bp_c, _ = B.fupr_prune(prod, Wp, bp, mask, [], [])
            folded[ci] = [Wp_c, bp_c]
            masks[(bi, ci)] = mask
            keeps[(bi, ci)] = keep
        sc = blk["shortcut"]
        proj_layer = None
        cat = None
        if sc["kind"] == "projection":
            Wf, bf = _fold(sc["conv"], sc["bn"])
            Wl = folded[-1][0]
            if (concat_projection and model["dtype"] != "f32" and Wl.shape[2:] == (1, 1)
                    and convs[-1]["stride"] == 1 and (bi, len(folded) - 1) not in keeps):
                cat = (B.shape_of(Wf, sc["conv"]["stride"], sc["conv"]["pad"]), Wf, bf)
            else:
                layers.append(Layer(f"b{bi}.proj", Wf, bf, sc["conv"]["stride"], sc["conv"]["pad"], False))
                proj_layer = len(layers) - 1
        first = len(layers)
        for ci, (Wf, bf) in enumerate(folded):
            last = ci == len(folded) - 1
            keep = keeps.get((bi, ci)) if last else None
            if last and cat is not None:
                sh_last = B.shape_of(Wf, convs[ci]["stride"], convs[ci]["pad"])
                _, Wc, bc = B.fupr_proj_concat(sh_last, Wf, bf, cat[0], cat[1], cat[2])
                layers.append(Layer(f"b{bi}.conv{ci + 1}+proj", Wc, bc, 1, 0, True,
                                    cat_stride=cat[0].stride))
                continue
            if keep is not None and Wf.shape[2] == 1 and Wf.shape[3] == 1:
                # A 1 x 1 last convolution is bound by writing the block's full-width output,
                # which removing filters does not shrink: its removed filters go back in as
                # zero rows (exact copies of the kept ones, zeros elsewhere), and the layer
                # runs as an ordinary convolution with the shortcut in its epilogue.
                k_full = convs[ci]["W"].shape[0]
                W_full = np.zeros((k_full,) + Wf.shape[1:], dtype=np.float32)
                b_full = np.zeros(k_full, dtype=np.float32)
                W_full[keep] = Wf
                b_full[keep] = bf
                Wf, bf, keep = W_full, b_full, None
            layers.append(Layer(f"b{bi}.conv{ci + 1}", Wf, bf, convs[ci]["stride"], convs[ci]["pad"],
                                True, add=last and sc["kind"] != "none", keep=keep))
        wiring.append(("block", (proj_layer, first, len(folded)), sc))
    head = model["head"]
    if head is not None:
        wiring.append(("avgpool", None, None))
        Wfc = np.ascontiguousarray(head["fc_W"][:, :, None, None], dtype=np.float32)
        layers.append(Layer("fc", Wfc, np.asarray(head["fc_b"], dtype=np.float32), 1, 0, False))
        wiring.append(("conv", len(layers) - 1, None))
    return {"layers": layers, "masks": masks, "keep_idx": keeps, "wiring": wiring,
            "dt": B.DTYPES[model["dtype"]], "in_shape": model["in_shape"]}


def build(plan, device="cuda:0", base_address=None):
    """Pack every layer, upload one blob, create the fupr model.

    base_address: plan on the host only - nothing is uploaded, the operators point
    at that (never dereferenced) address, and the model can be queried but not run.

    Returns (Model, sites) where sites[i] is the convolution site name of
    operator i (None for pools)."""
    dt = plan["dt"]
    blobs, offsets, total = [], [], 0
    for L in plan["layers"]:
        blob = B.fupr_pack(L.shape, L.W, L.bias, dt)
        offsets.append(total)
        blobs.append(blob)
        total += (len(blob) + 255) // 256 * 256
    keep_offsets = {}
    for li, L in enumerate(plan["layers"]):
        if L.keep is not None:
            keep_offsets[li] = total
            total += (4 * len(L.keep) + 255) // 256 * 256
    host = np.zeros(total, dtype=np.uint8)
    for off, blob in zip(offsets, blobs):
        host[off:off + len(blob)] = blob
    for li, off in keep_offsets.items():
        idx = np.ascontiguousarray(plan["layers"][li].keep, dtype=np.int32)
        host[off:off + 4 * len(idx)] = idx.view(np.uint8)
    dev = None if base_address is not None else B.upload_blob(host, device)
    base = base_address if dev is None else dev.data_ptr()

    ops, sites = [], []

    def conv_op(li, tin, res=-1, rss=1, roff=0, tin2=-1):
        L = plan["layers"][li]
        epi = (B.FUSE_RELU if L.relu else 0) | (B.FUSE_ADD if res >= 0 else 0)
        keep_ptr = None
        if L.keep is not None:
            epi |= B.FUSE_SCATTER
            keep_ptr = base + keep_offsets[li]
        if L.cat_stride:
            epi |= B.FUSE_CAT
        ops.append(B.OpDesc(B.OP_CONV, tin, res, L.shape, base + offsets[li], epi, rss, roff,
                            keep_ptr, tin2, max(L.cat_stride, 0)))
        sites.append(L.site)
        return len(ops)

    cur = 0
    for kind, a, sc in plan["wiring"]:
        if kind == "conv":
            cur = conv_op(a, cur)
        elif kind == "maxpool":
            k, st, pd = a
            ops.append(B.OpDesc(B.OP_MAXPOOL, cur, -1, B.conv_shape(1, 1, k, k, st, pd), None, 0, 1, 0))
            sites.append(None)
            cur = len(ops)
        elif kind == "avgpool":
            ops.append(B.OpDesc(B.OP_AVGPOOL, cur, -1, B.conv_shape(1, 1, 1, 1, 1, 0), None, 0, 1, 0))
            sites.append(None)
            cur = len(ops)
        else:
            proj, first, n = a
            x = cur
            res, rss = x, 1
            if sc["kind"] == "none":
                res = -1
            elif sc["kind"] == "optionA":
                rss = sc["stride"]
            # Where the projection shortcut goes in the operator list: the library runs a
            # block's last 1 x 1 convolution and the next block's first one as one kernel
            # when they are adjacent, so a bottleneck block's projection follows its first
            # convolution; a basic block's comes first.
            late = proj is not None and n >= 3
            if proj is not None and not late:
                res = conv_op(proj, x)
            h = x
            for i in range(n - 1):
                h = conv_op(first + i, h)
                if i == 0 and late:
                    res = conv_op(proj, x)
            if plan["layers"][first + n - 1].cat_stride:
                # the projection shortcut is part of the last convolution: it reads the block input
                cur = conv_op(first + n - 1, h, tin2=x)
            else:
                cur = conv_op(first + n - 1, h, res, rss, 0)
    model = B.Model(dt, plan["in_shape"], ops, keepalive=[dev], device=device)
    model.sites = sites
    model.plan = plan
    return model, sites
