"""GPU parity of MERGED_XCD and of its way out of a wait: stage 1 and the merged K x K GEMM in one launch, with a barrier
among the workgroups of each XCD in between.

Every case prints its name before it touches the GPU, so that a fault names its case.
"""
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.workloads import Layer, make_inputs
from parity_util import assert_parity

pytestmark = pytest.mark.gpu


def _announce(*parts):
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def _oracle(orc, layer, inputs):
    y, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
    return y


def _conv(layer, tuning, layout):
    from paper_2211_03715_amd.layer import TuckerConv2d
    return TuckerConv2d(layer, 0, B.make_tuning(variant=B.VARIANT_MERGED_XCD, **tuning), layout=layout)


def _tensors(inputs, layout):
    import torch
    dev = torch.device("cuda:0")
    t = {k: torch.from_numpy(v).to(dev) for k, v in inputs.items()}
    t["x"] = t["x"].permute(0, 2, 3, 1).contiguous() if layout == B.LAYOUT_NHWC else t["x"]
    return t


def _to_nchw(y, layout):
    return np.ascontiguousarray(y.transpose(0, 3, 1, 2)) if layout == B.LAYOUT_NHWC else y


# (stage-1 split, merged-GEMM split): every team size, including teams larger than a unit has k-groups
SPLITS = [(1, 1), (2, 8), (8, 2), (4, 4), (8, 8), (1, 8), (8, 1)]
LAYERS = [
    Layer(1, 256, 256, 14, 14, 64, 64),          # the 14x14 layer of the batch-1 configuration: one pass, 208 workgroups
    Layer(1, 512, 512, 7, 7, 128, 128),          # its 7x7 layer: 256 workgroups
    Layer(2, 20, 64, 19, 23, 32, 57),            # ragged everything, batch 2, several passes
    Layer(3, 33, 72, 12, 40, 8, 40, 3, 2, 1),    # stride 2, N % 16 != 0, batch 3
    Layer(1, 3, 2, 1, 1, 1, 1, 1, 1, 0),         # a single pixel: most workgroups have nothing to do and still must arrive
    Layer(1, 10, 12, 15, 17, 6, 5, 7, 1, 3),     # 7x7 taps
    Layer(1, 128, 128, 28, 28, 32, 32),          # 98 stage-1 units per XCD: more than one pass at every split
]


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("split", SPLITS, ids=lambda s: "k%d-%d" % s)
@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: l.name())
def test_forced_splits(orc, layer, split, layout):
    import torch
    if layout == B.LAYOUT_NHWC and (layer.C % 4 or layer.N % 4):
        pytest.skip("NHWC needs C and N in multiples of 4")
    _announce("merged_xcd", layer.name(), split, "nhwc" if layout else "nchw")
    inputs = make_inputs(layer, 4242)
    want = _oracle(orc, layer, inputs)
    conv = _conv(layer, dict(waves=(split[0], split[1], split[1])), layout)
    try:
        t = _tensors(inputs, layout)
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.full(conv.out_shape(), float("nan"), device="cuda:0")
        conv(t["x"], y)
        torch.cuda.synchronize()
        assert B.tdc_plan_status(conv.plan) == B.TDC_OK
        assert conv.kernel_count() == 1
        assert_parity(_to_nchw(y.cpu().numpy(), layout), want, "%s [%s]" % (layer.name(), conv.describe()))
    finally:
        conv.close()


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
def test_many_calls_and_graph_replays_agree(orc, layout):
    """The arrival words count calls on the device: 300 eager calls, then a captured graph replayed with eager calls
    and synchronisations in between, all give the first call's y bit for bit."""
    import torch
    layer = Layer(1, 256, 256, 14, 14, 64, 64)
    _announce("merged_xcd repeat + graph", layer.name(), "nhwc" if layout else "nchw")
    inputs = make_inputs(layer, 77)
    want = _oracle(orc, layer, inputs)
    conv = _conv(layer, {}, layout)
    try:
        t = _tensors(inputs, layout)
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y0 = torch.full(conv.out_shape(), float("nan"), device="cuda:0")
        conv(t["x"], y0)
        torch.cuda.synchronize()
        assert_parity(_to_nchw(y0.cpu().numpy(), layout), want, conv.describe())
        y = torch.empty_like(y0)
        for i in range(300):
            if i % 50 == 0:
                y.fill_(float("nan"))
            conv(t["x"], y)
            if i % 50 == 49:
                torch.cuda.synchronize()
                assert torch.equal(y, y0), "call %d differs" % i
        s = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        yg = torch.empty_like(y0)
        with torch.cuda.stream(s):
            launch = conv.bind(t["x"], yg, stream=s.cuda_stream)
            launch()
            s.synchronize()
            with torch.cuda.graph(g, stream=s):
                launch()
                launch()
        for rep in range(4):
            yg.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(yg, y0), "replay %d differs" % rep
            conv(t["x"], y)          # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(y, y0)
        assert B.tdc_plan_status(conv.plan) == B.TDC_OK
    finally:
        conv.close()


def test_epilogue(orc):
    import torch
    layer = Layer(2, 20, 64, 19, 23, 32, 57)
    _announce("merged_xcd epilogue", layer.name())
    inputs = make_inputs(layer, 5)
    rng = np.random.default_rng(5)
    want = _oracle(orc, layer, inputs)
    bias = rng.standard_normal(layer.N).astype(np.float32)
    res = rng.standard_normal(want.shape).astype(np.float32)
    want = np.maximum(want + bias[None, :, None, None].astype(np.float64) + res.astype(np.float64), 0.0)
    for layout in (B.LAYOUT_NCHW, B.LAYOUT_NHWC):
        conv = _conv(layer, dict(waves=(4, 8, 8)), layout)
        try:
            t = _tensors(inputs, layout)
            conv.pack(t["U_in"], t["core"], t["U_out"])
            r = torch.from_numpy(res).cuda()
            r = r.permute(0, 2, 3, 1).contiguous() if layout else r
            y = torch.full(conv.out_shape(), float("nan"), device="cuda:0")
            conv(t["x"], y, bias=torch.from_numpy(bias).cuda(), residual=r, relu=True)
            torch.cuda.synchronize()
            assert_parity(_to_nchw(y.cpu().numpy(), layout), want, conv.describe())
        finally:
            conv.close()


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("layer", [Layer(1, 256, 256, 14, 14, 64, 64), Layer(2, 20, 64, 19, 23, 32, 57),
                                   Layer(1, 128, 128, 28, 28, 32, 32)], ids=lambda l: l.name())
def test_workgroups_that_stop_waiting_compute_stage_1_themselves(orc, layer, layout):
    """With a poll limit of zero every workgroup that is not the last of its XCD to arrive stops waiting at once and
    computes all of stage 1 itself, while the others are still writing the same cells: the result must be the oracle's,
    bit-identical to the call that waited, and the plan counts the waits given up."""
    import torch
    _announce("merged_xcd wait limit 0", layer.name(), "nhwc" if layout else "nchw")
    inputs = make_inputs(layer, 9)
    want = _oracle(orc, layer, inputs)
    conv = _conv(layer, {}, layout)
    try:
        t = _tensors(inputs, layout)
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y0 = torch.full(conv.out_shape(), float("nan"), device="cuda:0")
        conv(t["x"], y0)
        torch.cuda.synchronize()
        assert B.tdc_plan_waits_given_up(conv.plan) == 0
        assert_parity(_to_nchw(y0.cpu().numpy(), layout), want, conv.describe())
        B.tdc_plan_set_wait_limit(conv.plan, 0)
        y = torch.empty_like(y0)
        for rep in range(5):
            y.fill_(float("nan"))
            conv(t["x"], y)
            torch.cuda.synchronize()
            assert B.tdc_plan_status(conv.plan) == B.TDC_OK
            assert torch.equal(y, y0), "call %d with the wait cut short differs" % rep
        assert B.tdc_plan_waits_given_up(conv.plan) > 0
        B.tdc_plan_set_wait_limit(conv.plan, 512)
        y.fill_(float("nan"))
        conv(t["x"], y)
        torch.cuda.synchronize()
        assert torch.equal(y, y0)
    finally:
        conv.close()


def test_two_plans_in_flight_on_two_streams(orc):
    """Two one-launch plans of 256 and 208 workgroups launched alternately on two streams: whether or not both launches
    are resident at once, every call must finish (a workgroup that waits too long goes on alone) and be right."""
    import torch
    la, lb = Layer(1, 512, 512, 7, 7, 128, 128), Layer(1, 256, 256, 14, 14, 64, 64)
    _announce("merged_xcd two streams", la.name(), lb.name())
    ia, ib = make_inputs(la, 21), make_inputs(lb, 22)
    wa, wb = _oracle(orc, la, ia), _oracle(orc, lb, ib)
    ca, cb = _conv(la, {}, B.LAYOUT_NCHW), _conv(lb, {}, B.LAYOUT_NCHW)
    try:
        ta, tb = _tensors(ia, B.LAYOUT_NCHW), _tensors(ib, B.LAYOUT_NCHW)
        ca.pack(ta["U_in"], ta["core"], ta["U_out"])
        cb.pack(tb["U_in"], tb["core"], tb["U_out"])
        ya = torch.full(ca.out_shape(), float("nan"), device="cuda:0")
        yb = torch.full(cb.out_shape(), float("nan"), device="cuda:0")
        torch.cuda.synchronize()
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        launch_a, launch_b = ca.bind(ta["x"], ya, stream=sa.cuda_stream), cb.bind(tb["x"], yb, stream=sb.cuda_stream)
        for _ in range(200):
            launch_a()
            launch_b()
        torch.cuda.synchronize()
        assert B.tdc_plan_status(ca.plan) == B.TDC_OK and B.tdc_plan_status(cb.plan) == B.TDC_OK
        assert_parity(ya.cpu().numpy(), wa, ca.describe())
        assert_parity(yb.cpu().numpy(), wb, cb.describe())
        print("    waits given up: %d and %d of 200 calls each" % (B.tdc_plan_waits_given_up(ca.plan), B.tdc_plan_waits_given_up(cb.plan)), flush=True)
    finally:
        ca.close()
        cb.close()


def test_next_to_launches_that_fill_the_gpu(orc):
    """A one-launch plan on one stream while batch-128 calls of 256 large workgroups keep the compute units busy from another:
    its workgroups become resident a few at a time, waits may run out, and every call must still be right."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    small, big = Layer(1, 512, 512, 7, 7, 128, 128), Layer(128, 128, 128, 28, 28, 32, 32)
    _announce("merged_xcd beside a full GPU", small.name(), big.name())
    i_small, i_big = make_inputs(small, 31), make_inputs(big, 32)
    want = _oracle(orc, small, i_small)
    c_small = _conv(small, {}, B.LAYOUT_NCHW)
    c_big = TuckerConv2d(big, 0, None)
    try:
        ts, tb = _tensors(i_small, B.LAYOUT_NCHW), _tensors(i_big, B.LAYOUT_NCHW)
        c_small.pack(ts["U_in"], ts["core"], ts["U_out"])
        c_big.pack(tb["U_in"], tb["core"], tb["U_out"])
        y_small = torch.full(c_small.out_shape(), float("nan"), device="cuda:0")
        y_big = torch.empty(c_big.out_shape(), device="cuda:0")
        torch.cuda.synchronize()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        l_small, l_big = c_small.bind(ts["x"], y_small, stream=s1.cuda_stream), c_big.bind(tb["x"], y_big, stream=s2.cuda_stream)
        for rep in range(3):
            y_small.fill_(float("nan"))
            torch.cuda.synchronize()
            for _ in range(60):
                l_big()
                l_small()
            torch.cuda.synchronize()
            assert B.tdc_plan_status(c_small.plan) == B.TDC_OK
            assert_parity(y_small.cpu().numpy(), want, "repeat %d %s" % (rep, c_small.describe()))
        print("    waits given up: %d in 180 calls" % B.tdc_plan_waits_given_up(c_small.plan), flush=True)
    finally:
        c_small.close()
        c_big.close()


def test_refusals():
    s = B.make_shape(1, 256, 256, 14, 14, 64, 64)
    for bad in (dict(waves=(3, 8, 8)), dict(waves=(8, 8, 8), mb=(2, 1, 1)), dict(waves=(8, 8, 8), pb=(1, 2, 2))):
        with pytest.raises(B.TdcError) as err:
            B.tdc_plan_create(s, 0, B.make_tuning(variant=B.VARIANT_MERGED_XCD, **bad))
        assert err.value.status == B.TDC_ERR_BAD_TUNING
    plan = B.tdc_plan_create(s, 0, B.make_tuning(variant=B.VARIANT_MERGED))
    try:
        assert B.tdc_plan_status(plan) == B.TDC_OK
        with pytest.raises(B.TdcError):
            B.tdc_plan_set_wait_limit(plan, 5)
    finally:
        B.tdc_plan_destroy(plan)
