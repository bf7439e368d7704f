"""GPU test of fupr_forward_static, the forward pass for callers that cannot
allocate device memory: through the C ABI, against fupr_forward on the same
inputs, two calls in a row, the second on a smaller batch."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fx():
    import torch
    from paper_2010_16165_amd import binding as B, network
    assert torch.cuda.is_available()
    return B, network, torch


def models():
    return [
        # one kernel per launch group: every intermediate tensor lives in the workspace
        ("imagenet basic", synth.make_imagenet_basic_resnet(51, "bf16", (1, 2, 1, 1), 300,
                                                            widths=(64, 16, 24, 40), size=64, classes=9), 6, 2),
        ("imagenet bottleneck", synth.make_imagenet_bottleneck_resnet(52, "f16", (2, 1, 1, 1), 500,
                                                                      widths=(16, 16, 24, 24), size=64,
                                                                      classes=5), 5, 3),
        # the one-kernel schedule (no workspace use at all) and its per-operator form
        ("cifar", synth.make_cifar_resnet(53, "bf16", 2, 400), 7, 4),
    ]


@pytest.mark.parametrize("mi", range(3))
def test_static_workspace_forward_equals_forward(fx, mi):
    B, network, torch = fx
    name, model, n_first, n_second = models()[mi]
    dt = B.DTYPES[model["dtype"]]
    m, _ = network.build(network.optimise(model))
    for schedule in (B.SCHEDULE_AUTO, B.SCHEDULE_PER_LAYER):
        m.set_schedule(schedule)
        for n in (n_first, n_second):          # two calls in a row, the second smaller
            print(f"{name}: schedule {schedule}, batch {n}", flush=True)
            assert m.workspace_bytes(n) <= B.fupr_static_workspace_bytes()
            x = synth.make_input(500 + n, n, model["in_shape"])
            xd = B.DeviceTensor.from_nchw(x, dt)
            want, ws = m.alloc(n)
            want.data.fill_(float("nan"))
            m.fupr_forward(xd, want, ws)
            torch.cuda.synchronize()
            got = B.DeviceTensor.empty(*want.data.shape[:3], want.C, dt, want.data.shape[3])
            got.data.fill_(float("nan"))
            m.fupr_forward_static(xd, got)
            torch.cuda.synchronize()
            assert torch.isfinite(got.data.float()).all()
            assert torch.equal(got.data, want.data)      # same kernels, same order: same bits


def test_static_workspace_refuses_what_does_not_fit(fx):
    B, network, torch = fx
    model = synth.make_imagenet_basic_resnet(51, "bf16", (1, 1, 1, 1), 300, widths=(64, 16, 24, 40),
                                             size=64, classes=9)
    m, _ = network.build(network.optimise(model))
    n = 1
    while m.workspace_bytes(n) <= B.fupr_static_workspace_bytes():
        n *= 2
    xd = B.DeviceTensor.empty(n, 64, 64, 3, B.BF16)
    out, _ = m.alloc(n)
    out.data.fill_(3.0)
    with pytest.raises(B.FuprError) as e:
        m.fupr_forward_static(xd, out)
    assert e.value.status == B.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out.data == 3.0).all())
    xs, ys = xd.struct, out.struct
    assert B._lib.fupr_forward_static(None, B.C.byref(xs), B.C.byref(ys), None) == B.ERR_NULL
