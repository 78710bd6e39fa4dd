"""GPU parity of the NHWC activation layout (tdc_shape.layout = 1) against the oracle.

The oracle works in NCHW; NHWC is the same tensor stored pixel-major, so the test permutes the
oracle's input and expected output (numpy transposes, no arithmetic) and everything else -- the
weights, the tolerance, the kernels' tunings -- is as in the NCHW tests."""
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.workloads import Layer, config_layers, layer_seed, make_dense_inputs, make_inputs
from parity_util import assert_parity

pytestmark = pytest.mark.gpu

VARIANTS = {"naive": B.VARIANT_NAIVE, "split": B.VARIANT_SPLIT, "fused": B.VARIANT_FUSED, "chain": B.VARIANT_CHAIN,
            "merged": B.VARIANT_MERGED, "fused_merged": B.VARIANT_FUSED_MERGED, "merged_xcd": B.VARIANT_MERGED_XCD,
            "auto": B.VARIANT_AUTO}

# C and N multiples of 4 (the layout's requirement), everything else ragged
SMALL = [
    Layer(1, 4, 8, 6, 9, 3, 4),
    Layer(2, 20, 24, 19, 23, 17, 33),           # C, N not multiples of 16: partial channel groups at both ends
    Layer(1, 64, 64, 56, 56, 16, 16),           # the primary case
    Layer(3, 36, 20, 12, 40, 8, 40, 3, 2, 1),   # stride 2, asymmetric ranks, batch 3
    Layer(1, 16, 16, 9, 9, 16, 16, 3, 1, 0),    # no padding
    Layer(2, 12, 12, 7, 5, 4, 6, 1, 1, 0),      # 1x1 core
    Layer(1, 8, 8, 11, 13, 5, 3, 5, 1, 2),      # 5x5 core
    Layer(1, 4, 4, 1, 1, 1, 1, 1, 1, 0),        # a single pixel
    Layer(1, 40, 24, 16, 16, 32, 48, 3, 2, 1),
    Layer(1, 12, 12, 15, 17, 6, 5, 7, 1, 3),    # 7x7 core: the largest stencil the library takes
    Layer(2, 8, 8, 18, 21, 4, 7, 7, 4, 6),      # ... with the largest stride (4) and padding (K - 1)
]


def _announce(*parts):
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def _run(layer, inputs, tuning=None, pack=True, epilogue=None):
    """One NHWC call on cuda:0; returns (y as numpy in NHWC, plan description)."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    dev = torch.device("cuda:0")
    t = {k: torch.from_numpy(nhwc(v) if k == "x" else v).to(dev) for k, v in inputs.items()}
    conv = TuckerConv2d(layer, 0, tuning, layout=B.LAYOUT_NHWC)
    try:
        if pack:
            conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        kw = {}
        if epilogue:
            kw = dict(bias=torch.from_numpy(epilogue["bias"]).to(dev), residual=torch.from_numpy(nhwc(epilogue["residual"])).to(dev),
                      relu=True)
        conv(t["x"], y, weights=(t["U_in"], t["core"], t["U_out"]), **kw)
        torch.cuda.synchronize()
        return y.cpu().numpy(), conv.describe()
    finally:
        conv.close()


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("layer", SMALL, ids=lambda l: l.name())
def test_nhwc_small_shapes(orc, variant, layer):
    _announce("nhwc small", variant, layer.name())
    inputs = make_inputs(layer, 4321)
    want, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
    got, desc = _run(layer, inputs, B.make_tuning(variant=VARIANTS[variant]))
    e = assert_parity(got, nhwc(want), "nhwc %s %s [%s]" % (variant, layer.name(), desc))
    print("   ", desc, "E_inf=%.2e E_el=%.2e" % e, flush=True)


FORCED = [
    ("fused_8x8_w4", dict(variant=B.VARIANT_FUSED, tile_h=8, tile_w=8, waves=(4, 4, 4), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("fused_4x16_w8_pb2", dict(variant=B.VARIANT_FUSED, tile_h=4, tile_w=16, waves=(8, 8, 8), mb=(2, 2, 4), pb=(2, 2, 2))),
    ("chain_4x12_w4", dict(variant=B.VARIANT_CHAIN, tile_h=4, tile_w=12, waves=(4, 4, 4), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("chain_7x7_w8_pb2", dict(variant=B.VARIANT_CHAIN, tile_h=7, tile_w=7, waves=(8, 8, 8), mb=(2, 2, 2), pb=(2, 2, 2))),
    ("fm_2x8_w4", dict(variant=B.VARIANT_FUSED_MERGED, tile_h=2, tile_w=8, waves=(4, 0, 0), mb=(1, 2, 0))),
    ("fm_4x4_w8_ks4", dict(variant=B.VARIANT_FUSED_MERGED, tile_h=4, tile_w=4, waves=(8, 0, 0), mb=(2, 2, 0))),
    ("split_w8", dict(variant=B.VARIANT_SPLIT, waves=(8, 8, 8), mb=(2, 2, 2), pb=(2, 2, 2))),
    ("merged_w1", dict(variant=B.VARIANT_MERGED, waves=(1, 1, 1), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("merged_w6_pb4", dict(variant=B.VARIANT_MERGED, waves=(6, 6, 6), mb=(1, 2, 2), pb=(4, 2, 2))),
]


@pytest.mark.parametrize("name,tuning", FORCED, ids=[f[0] for f in FORCED])
@pytest.mark.parametrize("layer", [Layer(2, 20, 64, 19, 23, 32, 32), Layer(1, 128, 128, 28, 28, 32, 32)], ids=lambda l: l.name())
def test_nhwc_forced_tunings(orc, name, tuning, layer):
    _announce("nhwc forced", name, layer.name())
    inputs = make_inputs(layer, 77)
    want, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
    got, desc = _run(layer, inputs, B.make_tuning(**tuning))
    assert_parity(got, nhwc(want), "nhwc %s %s [%s]" % (name, layer.name(), desc))
    got2, _ = _run(layer, inputs, B.make_tuning(**tuning), pack=False)      # weights re-laid out on every call
    assert np.array_equal(got, got2)


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("layer", [Layer(2, 20, 24, 19, 23, 17, 33), Layer(2, 32, 40, 8, 12, 16, 16)], ids=lambda l: l.name())
def test_nhwc_epilogue(orc, variant, layer):
    """bias + residual (laid out like y) + ReLU in the NHWC store of every kernel family."""
    _announce("nhwc epilogue", variant, layer.name())
    inputs = make_inputs(layer, 11)
    rng = np.random.default_rng(12)
    epi = dict(bias=rng.standard_normal(layer.N, dtype=np.float32),
               residual=rng.standard_normal((layer.batch, layer.N, layer.Ho, layer.Wo), dtype=np.float32))
    want, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
    want = orc.apply_epilogue(want, epi["bias"], epi["residual"], True)
    got, desc = _run(layer, inputs, B.make_tuning(variant=VARIANTS[variant]), epilogue=epi)
    assert_parity(got, nhwc(want), "nhwc epilogue %s %s [%s]" % (variant, layer.name(), desc))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6, 7])
def test_nhwc_full_size_workloads(orc, cfg):
    """All five workloads at full size with the selector's choice."""
    for i, layer in enumerate(config_layers(cfg)):
        _announce("nhwc config", cfg, "layer", i, layer.name())
        inputs = make_inputs(layer, layer_seed(cfg, i))
        want, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
        got, desc = _run(layer, inputs, None)
        e = assert_parity(got, nhwc(want), "nhwc config %d layer %d %s [%s]" % (cfg, i, layer.name(), desc))
        print("   ", desc, "E_inf=%.2e E_el=%.2e" % e, flush=True)


def test_nhwc_dense_layer(orc):
    import torch
    from paper_2211_03715_amd.layer import DenseConv2d
    dev = torch.device("cuda:0")
    for layer, tuning in ((Layer(2, 40, 64, 19, 23, 1, 1), None), (Layer(1, 20, 36, 14, 14, 1, 1, 3, 2, 1), dict(mb=(0, 1, 0), pb=(0, 2, 0), waves=(0, 4, 0))),
                          (Layer(1, 128, 128, 28, 28, 1, 1), None)):
        _announce("nhwc dense", layer.name(), tuning)
        inputs = make_dense_inputs(layer, 31)
        rng = np.random.default_rng(32)
        bias = rng.standard_normal(layer.N, dtype=np.float32)
        res = rng.standard_normal((layer.batch, layer.N, layer.Ho, layer.Wo), dtype=np.float32)
        want, _ = orc.conv_dense_with(orc.Shape(**layer.asdict()), inputs["x"], inputs["W"].astype(np.float64))
        conv = DenseConv2d(layer, 0, B.make_tuning(**tuning) if tuning else None, layout=B.LAYOUT_NHWC)
        try:
            x, W = torch.from_numpy(nhwc(inputs["x"])).to(dev), torch.from_numpy(inputs["W"]).to(dev)
            conv.pack(W)
            y = torch.full(conv.out_shape(), float("nan"), device=dev)
            conv(x, y)
            torch.cuda.synchronize()
            assert_parity(y.cpu().numpy(), nhwc(want), "nhwc dense %s [%s]" % (layer.name(), conv.describe()))
            y.fill_(float("nan"))
            conv(x, y, bias=torch.from_numpy(bias).to(dev), residual=torch.from_numpy(nhwc(res)).to(dev), relu=True)
            torch.cuda.synchronize()
            assert_parity(y.cpu().numpy(), nhwc(orc.apply_epilogue(want, bias, res, True)), "nhwc dense epilogue %s" % layer.name())
        finally:
            conv.close()


def test_nhwc_refusals():
    """Channel counts that are not multiples of 4 and misaligned tensors are refused, not mangled."""
    import torch
    for C, N in ((6, 8), (8, 6), (5, 7)):
        with pytest.raises(B.TdcError) as err:
            B.tdc_plan_create(B.make_shape(1, C, N, 8, 8, 2, 2, layout=B.LAYOUT_NHWC), 0)
        assert err.value.status == B.TDC_ERR_UNSUPPORTED
    with pytest.raises(B.TdcError) as err:
        B.tdc_plan_create(B.make_shape(1, 8, 8, 8, 8, 2, 2, layout=2), 0)
    assert err.value.status == B.TDC_ERR_UNSUPPORTED
    layer = Layer(1, 8, 8, 6, 6, 4, 4)
    _announce("nhwc misaligned", layer.name())
    lib = B.load()
    s = B.make_shape(**layer.asdict(), layout=B.LAYOUT_NHWC)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(v).cuda() for k, v in make_inputs(layer, 1).items()}
    xbuf = torch.zeros(8 * 36 + 4, device="cuda")
    ybuf = torch.zeros(8 * 36 + 4, device="cuda")
    plan = B.tdc_plan_create(s, 0)
    p = lambda a: a.data_ptr()
    try:
        assert lib.tdc_conv_tucker2(plan, st, p(xbuf) + 4, p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(ybuf), s) == B.TDC_ERR_UNSUPPORTED
        assert lib.tdc_conv_tucker2(plan, st, p(xbuf), p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(ybuf) + 8, s) == B.TDC_ERR_UNSUPPORTED
        assert lib.tdc_conv_tucker2(plan, st, p(xbuf), p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(ybuf), s) == B.TDC_OK
        torch.cuda.synchronize()
    finally:
        B.tdc_plan_destroy(plan)


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
def test_large_batch_sampled_images(orc, layout):
    """A batch far beyond the workloads' (200 images, 20 M elements each way): images are independent, so
    a few sampled images are compared with the oracle's result for that image alone."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    from dataclasses import replace
    layer = Layer(200, 128, 128, 28, 28, 32, 32)
    one = replace(layer, batch=1)
    _announce("large batch", layer.name(), "layout", layout)
    inputs = make_inputs(layer, 2025)
    dev = torch.device("cuda:0")
    x = inputs["x"] if layout == B.LAYOUT_NCHW else nhwc(inputs["x"])
    t = {k: torch.from_numpy(x if k == "x" else v).to(dev) for k, v in inputs.items()}
    conv = TuckerConv2d(layer, 0, None, layout=layout)
    try:
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        conv(t["x"], y)
        torch.cuda.synchronize()
        assert torch.isfinite(y).all()
        got = y.cpu().numpy()
        for b in (0, 1, 99, 198, 199):
            want, _ = orc.conv_factored(orc.Shape(**one.asdict()), inputs["x"][b:b + 1], inputs["U_in"], inputs["core"], inputs["U_out"])
            want = want if layout == B.LAYOUT_NCHW else nhwc(want)
            assert_parity(got[b:b + 1], want, "image %d of 200 [%s]" % (b, conv.describe()))
    finally:
        conv.close()


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
def test_one_image_at_the_size_limit(orc, layout):
    """The largest image the library accepts: 16 channels of 4096 x 8188 pixels, 2.146 GB each way, just under the
    2 GiB one buffer descriptor spans (byte offsets inside an image then use nearly all of 31 bits).  The
    convolution is local, so windows of the output -- the four corners, tile seams in the middle, the last rows --
    are compared with the oracle run on the matching crop of x (rows and columns next to a cut edge are left out:
    the oracle pads the crop with zeros there, the image does not)."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    layer = Layer(1, 16, 16, 4096, 8188, 8, 8)
    assert B.tdc_select_tuning(B.make_shape(**layer.asdict(), layout=layout)).variant in (B.VARIANT_FUSED, B.VARIANT_CHAIN)
    with pytest.raises(B.TdcError) as err:              # four more columns and an image no longer fits
        B.tdc_plan_create(B.make_shape(1, 16, 16, 4096, 8192, 8, 8, layout=layout), 0)
    assert err.value.status == B.TDC_ERR_UNSUPPORTED
    _announce("one image at the size limit", layer.name(), "layout", layout)
    inputs = make_inputs(layer, 4096)
    dev = torch.device("cuda:0")
    x_dev = torch.from_numpy(inputs["x"]).to(dev)
    if layout == B.LAYOUT_NHWC:
        x_dev = x_dev.permute(0, 2, 3, 1).contiguous()
    t = {k: torch.from_numpy(v).to(dev) for k, v in inputs.items() if k != "x"}
    conv = TuckerConv2d(layer, 0, None, layout=layout)
    try:
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        conv(x_dev, y)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(y).all()), "some outputs were never written"
        H, W = layer.H, layer.W
        windows = [(0, 40, 0, 72), (0, 40, W - 72, W), (H - 40, H, 0, 72), (H - 40, H, W - 72, W),
                   (2030, 2070, 4070, 4142), (H - 24, H, 3000, 3064), (1000, 1024, W - 64, W)]
        for (r0, r1, c0, c1) in windows:
            crop = np.ascontiguousarray(inputs["x"][:, :, r0:r1, c0:c1])
            small = Layer(1, layer.C, layer.N, r1 - r0, c1 - c0, layer.R1, layer.R2)
            want, _ = orc.conv_factored(orc.Shape(**small.asdict()), crop, inputs["U_in"], inputs["core"], inputs["U_out"])
            a, b = (1 if r0 > 0 else 0), (1 if r1 < H else 0)          # rows / columns spoiled by the cut
            c, d = (1 if c0 > 0 else 0), (1 if c1 < W else 0)
            want = want[:, :, a:want.shape[2] - b, c:want.shape[3] - d]
            if layout == B.LAYOUT_NCHW:
                got = y[:, :, r0 + a:r1 - b, c0 + c:c1 - d].cpu().numpy()
            else:
                got = y[:, r0 + a:r1 - b, c0 + c:c1 - d, :].permute(0, 3, 1, 2).contiguous().cpu().numpy()
            assert_parity(got, want, "window rows %d:%d cols %d:%d [%s]" % (r0, r1, c0, c1, conv.describe()))
    finally:
        conv.close()
