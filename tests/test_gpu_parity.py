"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by element.

Every case prints its name before it touches the GPU, so that a fault names its case.
"""
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.workloads import Layer, config_layers, layer_seed, make_inputs
from parity_util import assert_parity, run_gpu

pytestmark = pytest.mark.gpu

VARIANTS = {"naive": B.VARIANT_NAIVE, "split": B.VARIANT_SPLIT, "fused": B.VARIANT_FUSED, "chain": B.VARIANT_CHAIN,
            "merged": B.VARIANT_MERGED, "fused_merged": B.VARIANT_FUSED_MERGED, "merged_xcd": B.VARIANT_MERGED_XCD,
            "auto": B.VARIANT_AUTO}


def _announce(*parts):
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def _oracle(orc, layer, inputs):
    y, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
    return y


# Small shapes that still span several 16-wide blocks and ragged tails in every dimension.
SMALL = [
    Layer(1, 5, 7, 6, 9, 3, 4),                 # nothing a multiple of anything
    Layer(2, 20, 24, 19, 23, 17, 33),           # ranks just over a 16-block, odd image
    Layer(1, 64, 64, 56, 56, 16, 16),           # the primary case
    Layer(3, 33, 18, 12, 40, 8, 40, 3, 2, 1),   # stride 2, asymmetric ranks, batch 3
    Layer(1, 16, 16, 9, 9, 16, 16, 3, 1, 0),    # no padding
    Layer(2, 12, 10, 7, 5, 4, 6, 1, 1, 0),      # 1x1 core
    Layer(1, 8, 8, 11, 13, 5, 3, 5, 1, 2),      # 5x5 core
    Layer(1, 6, 9, 10, 10, 2, 2, 3, 3, 1),      # stride 3
    Layer(1, 3, 2, 1, 1, 1, 1, 1, 1, 0),        # a single pixel
    Layer(1, 4, 4, 3, 3, 2, 2, 3, 1, 1),        # image smaller than any tile
    Layer(1, 40, 24, 16, 16, 32, 48, 3, 2, 1),
    Layer(1, 10, 12, 15, 17, 6, 5, 7, 1, 3),    # 7x7 core: the largest stencil the library takes
    Layer(2, 9, 6, 18, 21, 4, 7, 7, 4, 6),      # ... with the largest stride (4) and padding (K - 1)
]


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("layer", SMALL, ids=lambda l: l.name())
def test_small_shapes(orc, variant, layer):
    _announce("small", variant, layer.name())
    inputs = make_inputs(layer, 1234)
    want = _oracle(orc, layer, inputs)
    got, desc = run_gpu(layer, inputs, B.make_tuning(variant=VARIANTS[variant]))
    e = assert_parity(got, want, "%s %s [%s]" % (variant, layer.name(), desc))
    print("   ", desc, "E_inf=%.2e E_el=%.2e" % e, flush=True)


FORCED = [
    ("fused_8x8_w4", dict(variant=B.VARIANT_FUSED, tile_h=8, tile_w=8, waves=(4, 4, 4), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("fused_4x16_w8", dict(variant=B.VARIANT_FUSED, tile_h=4, tile_w=16, waves=(8, 8, 8), mb=(2, 2, 4), pb=(1, 1, 1))),
    ("fused_7x7_w2_pb2", dict(variant=B.VARIANT_FUSED, tile_h=7, tile_w=7, waves=(2, 2, 2), mb=(2, 2, 2), pb=(2, 2, 2))),
    ("fused_3x5_w1", dict(variant=B.VARIANT_FUSED, tile_h=3, tile_w=5, waves=(1, 1, 1), mb=(4, 4, 4), pb=(2, 2, 2))),
    ("fused_16x32_w4", dict(variant=B.VARIANT_FUSED, tile_h=16, tile_w=32, waves=(4, 4, 4), mb=(4, 4, 4), pb=(1, 1, 1))),
    ("chain_8x8_w4", dict(variant=B.VARIANT_CHAIN, tile_h=8, tile_w=8, waves=(4, 4, 4), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("chain_4x28_w8_pb2", dict(variant=B.VARIANT_CHAIN, tile_h=4, tile_w=28, waves=(8, 8, 8), mb=(2, 1, 1), pb=(2, 2, 2))),
    ("chain_3x5_w1", dict(variant=B.VARIANT_CHAIN, tile_h=3, tile_w=5, waves=(1, 1, 1), mb=(4, 1, 1), pb=(2, 2, 2))),
    ("chain_7x7_w2", dict(variant=B.VARIANT_CHAIN, tile_h=7, tile_w=7, waves=(2, 2, 2), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("split_111_w1", dict(variant=B.VARIANT_SPLIT, waves=(1, 1, 1), mb=(1, 1, 1), pb=(1, 1, 1))),
    ("split_w8", dict(variant=B.VARIANT_SPLIT, waves=(8, 8, 8), mb=(1, 2, 4), pb=(4, 2, 1))),
    ("split_w3_44", dict(variant=B.VARIANT_SPLIT, waves=(3, 4, 2), mb=(4, 4, 4), pb=(4, 4, 4))),
    ("split_w2_24", dict(variant=B.VARIANT_SPLIT, waves=(2, 4, 1), mb=(2, 4, 2), pb=(1, 1, 2))),
]
FORCED_LAYERS = [Layer(2, 20, 60, 19, 23, 52, 64), Layer(1, 64, 64, 56, 56, 16, 16),
                 Layer(2, 33, 128, 12, 40, 32, 57, 3, 2, 1), Layer(1, 256, 256, 14, 14, 64, 64)]


@pytest.mark.parametrize("name,tuning", FORCED, ids=[f[0] for f in FORCED])
@pytest.mark.parametrize("layer", FORCED_LAYERS, ids=lambda l: l.name())
def test_forced_tunings(orc, name, tuning, layer):
    """Every register-tile shape, wave count and tile geometry the selector may pick."""
    _announce("forced", name, layer.name())
    inputs = make_inputs(layer, 77)
    blocks = [(layer.R1 + 15) // 16, (layer.R2 + 15) // 16, (layer.N + 15) // 16]
    if any(nb % mb for nb, mb in zip(blocks, tuning["mb"])):
        # register tiles must divide the channel blocks: the library refuses, nothing runs
        with pytest.raises(B.TdcError) as err:
            run_gpu(layer, inputs, B.make_tuning(**tuning))
        assert err.value.status == B.TDC_ERR_BAD_TUNING
        return
    want = _oracle(orc, layer, inputs)
    try:
        got, desc = run_gpu(layer, inputs, B.make_tuning(**tuning))
    except B.TdcError as e:
        if e.status == B.TDC_ERR_BAD_TUNING and name == "fused_16x32_w4":
            pytest.skip("tile does not fit the LDS budget for this layer")   # the library said so, nothing ran
        raise
    assert_parity(got, want, "%s %s [%s]" % (name, layer.name(), desc))


MERGED_FORCED = [dict(waves=(1, 1, 1), mb=(1, 1, 1), pb=(1, 1, 1)), dict(waves=(8, 8, 8), mb=(1, 2, 2), pb=(4, 2, 2)),
                 dict(waves=(3, 4, 4), mb=(2, 4, 4), pb=(1, 1, 1)), dict(waves=(2, 6, 6), mb=(1, 1, 1), pb=(2, 4, 4))]


@pytest.mark.parametrize("tuning", MERGED_FORCED, ids=lambda t: "w%d-%d_mb%d-%d_pb%d-%d" % (
    t["waves"][0], t["waves"][1], t["mb"][0], t["mb"][1], t["pb"][0], t["pb"][1]))
@pytest.mark.parametrize("layer", [Layer(2, 20, 64, 19, 23, 32, 57), Layer(1, 256, 256, 14, 14, 64, 64),
                                   Layer(2, 33, 128, 12, 40, 32, 57, 3, 2, 1)], ids=lambda l: l.name())
def test_forced_merged_tunings(orc, tuning, layer):
    """Stage 1 and the merged stage-2/3 convolution with every register-tile shape."""
    _announce("forced merged", tuning, layer.name())
    inputs = make_inputs(layer, 78)
    want = _oracle(orc, layer, inputs)
    got, desc = run_gpu(layer, inputs, B.make_tuning(variant=B.VARIANT_MERGED, **tuning))
    assert_parity(got, want, "%s [%s]" % (layer.name(), desc))


FM_FORCED = [
    (Layer(1, 64, 64, 56, 56, 16, 16), dict(tile_h=1, tile_w=14, waves=(4, 0, 0), mb=(1, 4, 0))),          # no k-split
    (Layer(1, 128, 128, 28, 28, 32, 32), dict(tile_h=1, tile_w=14, waves=(8, 0, 0), mb=(2, 4, 0))),        # 2 slices
    (Layer(1, 256, 256, 14, 14, 64, 64), dict(tile_h=2, tile_w=14, waves=(8, 0, 0), mb=(1, 2, 0))),        # 4 slices, 2 pixel blocks
    (Layer(1, 256, 256, 14, 14, 64, 64), dict(tile_h=4, tile_w=14, waves=(4, 0, 0), mb=(4, 1, 0))),        # 4 pixel blocks, ragged tile rows
    (Layer(2, 33, 72, 12, 40, 32, 57, 3, 2, 1), dict(tile_h=4, tile_w=16, waves=(4, 0, 0), mb=(1, 1, 0))), # stride 2, N not a multiple of 16
    (Layer(2, 33, 80, 12, 40, 16, 57, 3, 2, 1), dict(tile_h=3, tile_w=10, waves=(5, 0, 0), mb=(1, 5, 0))), # five blocks per workgroup
    (Layer(1, 8, 8, 11, 13, 5, 3, 5, 1, 2), dict(tile_h=4, tile_w=13, waves=(4, 0, 0), mb=(1, 1, 0))),     # 5x5 taps
    (Layer(3, 20, 24, 19, 23, 17, 33), dict(tile_h=3, tile_w=7, waves=(6, 0, 0), mb=(1, 2, 0))),           # uneven slices (18 k-groups / 3)
]


@pytest.mark.parametrize("layer,tuning", FM_FORCED, ids=["%s_%dx%d_w%d_mb%d_nbg%d" % (
    l.name(), t["tile_h"], t["tile_w"], t["waves"][0], t["mb"][0], t["mb"][1]) for l, t in FM_FORCED])
def test_forced_fused_merged_tunings(orc, layer, tuning):
    """The one-launch kernel with contraction slices, several pixel blocks and channel-block groups."""
    _announce("forced fused_merged", tuning, layer.name())
    inputs = make_inputs(layer, 79)
    want = _oracle(orc, layer, inputs)
    got, desc = run_gpu(layer, inputs, B.make_tuning(variant=B.VARIANT_FUSED_MERGED, **tuning))
    assert_parity(got, want, "%s [%s]" % (layer.name(), desc))


def test_fused_merged_refuses_what_it_cannot_hold():
    """Ranks whose contraction slices exceed the fragments a wavefront keeps in registers are refused."""
    with pytest.raises(B.TdcError) as err:
        B.tdc_plan_create(B.make_shape(1, 512, 512, 7, 7, 152, 152), 0, B.make_tuning(variant=B.VARIANT_FUSED_MERGED))
    assert err.value.status == B.TDC_ERR_BAD_TUNING


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6, 7])
def test_full_size_workloads(orc, cfg):
    """Every layer of the synthetic workloads (the five stated ones and the throughput set) at full size, in the launch configuration the
    benchmark times (selector's choice, weights re-laid out once), compared element by element."""
    worst = (0.0, 0.0)
    for i, layer in enumerate(config_layers(cfg)):
        _announce("config", cfg, "layer", i, layer.name())
        inputs = make_inputs(layer, layer_seed(cfg, i))
        want = _oracle(orc, layer, inputs)
        got, desc = run_gpu(layer, inputs, None)
        e = assert_parity(got, want, "config %d layer %d %s [%s]" % (cfg, i, layer.name(), desc))
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        print("   ", desc, "E_inf=%.2e E_el=%.2e" % e, flush=True)
    print("[config %d] worst E_inf=%.2e E_el=%.2e" % ((cfg,) + worst), flush=True)


@pytest.mark.parametrize("variant", ["split", "fused", "chain", "merged", "fused_merged"])
def test_dense_path_agrees_too(orc, variant):
    """The GPU result also matches the dense convolution with the kernel of Eq. 1."""
    layer = Layer(1, 24, 20, 14, 14, 12, 9)
    _announce("dense", variant, layer.name())
    inputs = make_inputs(layer, 5)
    want, _ = orc.conv_dense(orc.Shape(**layer.asdict()), **inputs)
    got, desc = run_gpu(layer, inputs, B.make_tuning(variant=VARIANTS[variant]))
    assert_parity(got, want, desc)


@pytest.mark.parametrize("variant", ["naive", "split", "fused", "chain", "merged", "fused_merged"])
def test_unpacked_weights_path(orc, variant):
    """Without tdc_plan_pack_weights the library re-lays the weights out on every call."""
    layer = Layer(2, 20, 24, 19, 23, 17, 33)
    _announce("unpacked", variant, layer.name())
    inputs = make_inputs(layer, 9)
    want = _oracle(orc, layer, inputs)
    got, desc = run_gpu(layer, inputs, B.make_tuning(variant=VARIANTS[variant]), pack=False)
    assert_parity(got, want, desc)


def test_repacking_after_weight_change_and_determinism(orc):
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    layer = Layer(1, 64, 64, 28, 28, 16, 32)
    _announce("repack+determinism", layer.name())
    dev = torch.device("cuda:0")
    for variant in (B.VARIANT_SPLIT, B.VARIANT_FUSED, B.VARIANT_CHAIN):
        a = make_inputs(layer, 11)
        b = make_inputs(layer, 12)
        ta = {k: torch.from_numpy(v).to(dev) for k, v in a.items()}
        conv = TuckerConv2d(layer, 0, B.make_tuning(variant=variant))
        conv.pack(ta["U_in"], ta["core"], ta["U_out"])
        y0 = conv(ta["x"]).clone()
        for _ in range(10):   # no atomics anywhere: repeated runs are bit-identical
            assert torch.equal(conv(ta["x"]), y0)
        assert_parity(y0.cpu().numpy(), _oracle(orc, layer, a), conv.describe())
        # new weight values in the same buffers, then pack again
        for k in ("U_in", "core", "U_out"):
            ta[k].copy_(torch.from_numpy(b[k]))
        conv.pack(ta["U_in"], ta["core"], ta["U_out"])
        y1 = conv(ta["x"])
        torch.cuda.synchronize()
        assert_parity(y1.cpu().numpy(), _oracle(orc, layer, dict(b, x=a["x"])), conv.describe())
        conv.close()


def test_linearity_and_batch_independence_on_gpu(orc):
    layer = Layer(4, 32, 48, 14, 14, 16, 16)
    _announce("linearity/batch", layer.name())
    one = Layer(1, 32, 48, 14, 14, 16, 16)
    inputs = make_inputs(layer, 21)
    for variant in (B.VARIANT_SPLIT, B.VARIANT_FUSED, B.VARIANT_CHAIN):
        yb, _ = run_gpu(layer, inputs, B.make_tuning(variant=variant))
        for b in range(4):
            y1, _ = run_gpu(one, dict(inputs, x=inputs["x"][b:b + 1].copy()), B.make_tuning(variant=variant))
            assert_parity(y1[0], yb[b].astype(np.float64), "image %d" % b)
        y2, _ = run_gpu(layer, dict(inputs, x=(2.0 * inputs["x"]).astype(np.float32)), B.make_tuning(variant=variant))
        assert np.array_equal(y2, 2.0 * yb), "scaling x by 2 must scale y by exactly 2"


RUN_MAJOR_LAYERS = [
    Layer(40, 20, 24, 12, 16, 17, 33),            # ragged channels and ranks, image 12 x 16
    Layer(24, 33, 18, 24, 40, 8, 40, 3, 2, 1),    # stride 2
    Layer(64, 16, 16, 12, 12, 16, 16, 3, 1, 0),   # no padding: no column outside the image
    Layer(40, 8, 8, 12, 16, 5, 3, 5, 1, 2),       # 5x5 core, two columns of padding each side
    Layer(70, 12, 10, 8, 8, 4, 6, 1, 1, 0),       # 1x1 core
    Layer(1100, 4, 4, 2, 4, 2, 2, 3, 1, 1),       # an image of one run per row
]
RUN_MAJOR_TUNINGS = [
    dict(variant=B.VARIANT_FUSED, tile_h=3, tile_w=5, waves=(4, 4, 4), mb=(1, 1, 1), pb=(1, 1, 1)),     # tiles start off the 4-grid
    dict(variant=B.VARIANT_FUSED, tile_h=2, tile_w=16, waves=(8, 8, 8), mb=(1, 1, 1), pb=(2, 2, 2)),
    dict(variant=B.VARIANT_CHAIN, tile_h=4, tile_w=7, waves=(2, 2, 2), mb=(1, 1, 1), pb=(1, 1, 1)),
    dict(variant=B.VARIANT_CHAIN, tile_h=12, tile_w=4, waves=(8, 8, 8), mb=(1, 1, 1), pb=(2, 2, 2)),
    dict(variant=B.VARIANT_FUSED),
    dict(variant=B.VARIANT_CHAIN),
]


@pytest.mark.parametrize("tuning", RUN_MAJOR_TUNINGS, ids=lambda t: "%s_%dx%d" % (
    "fused" if t["variant"] == B.VARIANT_FUSED else "chain", t.get("tile_h", 0), t.get("tile_w", 0)))
@pytest.mark.parametrize("layer", RUN_MAJOR_LAYERS, ids=lambda l: l.name())
def test_run_major_stage1_shapes(orc, layer, tuning):
    """In the throughput regime (batch x output pixels fill the chip) the fused and chain kernels read NCHW
    rows whose width is a multiple of 4 in 16-byte runs: ragged shapes and tiles that start off the 4-pixel
    grid, at batch sizes that select that path."""
    assert layer.batch * layer.Ho * layer.Wo >= 4096 and layer.W % 4 == 0
    _announce("run-major", layer.name(), tuning)
    inputs = make_inputs(layer, 909)
    want = _oracle(orc, layer, inputs)
    try:
        got, desc = run_gpu(layer, inputs, B.make_tuning(**tuning))
    except B.TdcError as e:
        if e.status == B.TDC_ERR_BAD_TUNING and "tile_h" in tuning:
            pytest.skip("tile does not fit this layer")          # the library said so, nothing ran
        raise
    assert_parity(got, want, "%s [%s]" % (layer.name(), desc))


def test_run_major_refuses_misaligned_x(orc):
    """A plan that reads NCHW rows sixteen bytes at a time refuses an x that is not 16-byte aligned (status, nothing
    launched); the same plan on the aligned buffer matches the oracle."""
    import torch
    layer = RUN_MAJOR_LAYERS[0]
    _announce("run-major misaligned x", layer.name())
    lib = B.load()
    inputs = make_inputs(layer, 911)
    want = _oracle(orc, layer, inputs)
    t = {k: torch.from_numpy(v).cuda() for k, v in inputs.items()}
    n_x = t["x"].numel()
    xbuf = torch.zeros(n_x + 4, device="cuda")
    xbuf[:n_x] = t["x"].reshape(-1)
    y = torch.full((layer.batch, layer.N, layer.Ho, layer.Wo), float("nan"), device="cuda")
    s = B.make_shape(**layer.asdict())
    st = torch.cuda.current_stream().cuda_stream
    plan = B.tdc_plan_create(s, 0, B.make_tuning(variant=B.VARIANT_CHAIN))
    p = lambda a: a.data_ptr()
    try:
        assert lib.tdc_conv_tucker2(plan, st, p(xbuf) + 4, p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(y), s) == B.TDC_ERR_UNSUPPORTED
        torch.cuda.synchronize()
        assert bool(torch.isnan(y).all())                      # nothing was written
        assert lib.tdc_conv_tucker2(plan, st, p(xbuf), p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(y), s) == B.TDC_OK
        torch.cuda.synchronize()
        assert_parity(y.cpu().numpy(), want, "run-major, aligned call after a refused one")
    finally:
        B.tdc_plan_destroy(plan)


def test_chain_takes_a_y_that_is_only_4_byte_aligned(orc):
    """The NCHW CHAIN kernel writes y sixteen bytes at a time where rows allow it; a y that is only 4-byte aligned (a
    slice of a larger tensor) is not refused but written with 4-byte stores, and nothing outside it is touched."""
    import torch
    layer = Layer(2, 32, 40, 8, 12, 16, 16)                  # tile and image widths multiples of 4: the 16-byte store path
    _announce("chain, y 4-byte aligned", layer.name())
    lib = B.load()
    inputs = make_inputs(layer, 912)
    want = _oracle(orc, layer, inputs)
    t = {k: torch.from_numpy(v).cuda() for k, v in inputs.items()}
    n_y = layer.batch * layer.N * layer.Ho * layer.Wo
    ybuf = torch.full((n_y + 8,), float("nan"), device="cuda")
    s = B.make_shape(**layer.asdict())
    st = torch.cuda.current_stream().cuda_stream
    plan = B.tdc_plan_create(s, 0, B.make_tuning(variant=B.VARIANT_CHAIN, tile_h=4, tile_w=12, waves=(4, 4, 4), mb=(1, 1, 1), pb=(1, 1, 1)))
    p = lambda a: a.data_ptr()
    try:
        for shift in (1, 0):                                  # floats: 4-byte aligned only, then 16-byte aligned
            ybuf.fill_(float("nan"))
            rc = lib.tdc_conv_tucker2(plan, st, p(t["x"]), p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(ybuf) + 4 * shift, s)
            assert rc == B.TDC_OK, B.status_string(rc)
            torch.cuda.synchronize()
            got = ybuf[shift:shift + n_y].cpu().numpy().reshape(want.shape)
            assert_parity(got, want, "chain with y shifted by %d floats" % shift)
            rest = torch.cat([ybuf[:shift], ybuf[shift + n_y:]])
            assert bool(torch.isnan(rest).all())              # the floats around y were left alone
    finally:
        B.tdc_plan_destroy(plan)


def test_pack_on_one_stream_conv_on_another(orc):
    """layer.py orders a conv call behind a weight re-layout that was enqueued on another stream."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    layer = Layer(2, 64, 64, 28, 28, 16, 32)
    _announce("pack stream != conv stream", layer.name())
    inputs = make_inputs(layer, 913)
    want = _oracle(orc, layer, inputs)
    t = {k: torch.from_numpy(v).cuda() for k, v in inputs.items()}
    side = torch.cuda.Stream()
    for variant in (B.VARIANT_FUSED, B.VARIANT_MERGED):
        conv = TuckerConv2d(layer, 0, B.make_tuning(variant=variant))
        try:
            side.wait_stream(torch.cuda.current_stream())     # the weights were uploaded on the current stream
            for _ in range(3):
                conv.pack(t["U_in"], t["core"], t["U_out"], stream=side)
                y = conv(t["x"])                              # current stream
                torch.cuda.synchronize()
                assert_parity(y.cpu().numpy(), want, conv.describe())
        finally:
            conv.close()


def test_two_plans_on_two_streams(orc):
    """Calls only enqueue on the stream they are given: two layers with plans of their own run on two
    non-default streams at once, repeatedly, and each matches the oracle (no hidden use of the default stream,
    no workspace shared between plans)."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    dev = torch.device("cuda:0")
    cases = []
    for layer, variant, seed in ((Layer(1, 256, 256, 14, 14, 64, 64), B.VARIANT_MERGED, 5),
                                 (Layer(2, 64, 64, 28, 28, 16, 16), B.VARIANT_SPLIT, 6)):
        _announce("streams", layer.name(), variant)
        inputs = make_inputs(layer, seed)
        t = {k: torch.from_numpy(v).to(dev) for k, v in inputs.items()}
        conv = TuckerConv2d(layer, 0, B.make_tuning(variant=variant))
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        cases.append((conv, t, y, _oracle(orc, layer, inputs), torch.cuda.Stream()))
    torch.cuda.synchronize()
    try:
        for _ in range(20):
            for conv, t, y, _, stream in cases:
                conv(t["x"], y, stream=stream)
        for conv, t, y, want, stream in cases:
            stream.synchronize()
            assert_parity(y.cpu().numpy(), want, conv.describe())
    finally:
        for conv, *_ in cases:
            conv.close()


@pytest.mark.parametrize("share", [1, 2], ids=["planned_for_the_chip", "planned_for_half_the_chip"])
@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
def test_three_calls_in_flight_at_full_size(orc, layout, share):
    """The configuration bench.py's `concurrent` figures time: three plans of one batch-32 layer (the selector's choice
    for the whole chip or for half of its compute units, the one-launch kernels) on three streams, launched round-robin
    so that their workgroups share compute units; every call's output against the oracle on its own input."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    dev = torch.device("cuda:0")
    layer = Layer(32, 128, 128, 28, 28, 32, 32)
    _announce("three streams", layer.name(), "layout", layout)
    base = make_inputs(layer, 77)
    w = {k: torch.from_numpy(base[k]).to(dev) for k in ("U_in", "core", "U_out")}
    cases = []
    for seed in (78, 79, 80):
        inputs = dict(base, x=make_inputs(layer, seed)["x"])
        want = _oracle(orc, layer, inputs)
        x = torch.from_numpy(inputs["x"]).to(dev)
        if layout == B.LAYOUT_NHWC:
            x, want = x.permute(0, 2, 3, 1).contiguous(), np.ascontiguousarray(np.transpose(want, (0, 2, 3, 1)))
        tuning = B.tdc_select_tuning(B.make_shape(**layer.asdict(), layout=layout), compute_units=torch.cuda.get_device_properties(dev).multi_processor_count // share) if share > 1 else None
        conv = TuckerConv2d(layer, 0, tuning, layout=layout)
        conv.pack(w["U_in"], w["core"], w["U_out"])
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        stream = torch.cuda.Stream()
        torch.cuda.synchronize()
        cases.append((conv, conv.bind(x, y, stream=stream.cuda_stream), x, y, want, stream))
    try:
        for _ in range(30):
            for _, launch, *_ in cases:
                launch()
        for conv, _, _, y, want, stream in cases:
            stream.synchronize()
            assert_parity(y.cpu().numpy(), want, conv.describe())
    finally:
        for conv, *_ in cases:
            conv.close()


def _random_cases(n, seed):
    """Seeded random layers and one-launch tunings: batches of 1 to 9 images, tile counts and workgroup totals that are
    not multiples of the 8 XCDs the kernels renumber their workgroups over, every stage-1 width."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        K = int(rng.choice([1, 3, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 2]))
        pad = int(rng.integers(0, K))
        H, W = int(rng.integers(K, 30)), int(rng.integers(K, 34))
        C, N = int(rng.integers(1, 70)), int(rng.integers(1, 70))
        R1, R2 = int(rng.choice([4, 8, 16, 24, 32, 40, 64])), int(rng.choice([4, 8, 16, 24, 32, 48]))
        layer = Layer(int(rng.integers(1, 10)), C, N, H, W, R1, R2, K, stride, pad)
        if layer.Ho < 1 or layer.Wo < 1:
            continue
        variant = str(rng.choice(["fused", "chain", "fused_merged"]))
        nb1 = (R1 + 15) // 16
        mb1 = int(rng.choice([m for m in (1, 2, 4) if nb1 % m == 0]))
        tuning = dict(tile_h=int(rng.integers(1, min(layer.Ho, 8) + 1)), tile_w=int(rng.integers(1, min(layer.Wo, 16) + 1)),
                      waves=(int(rng.choice([1, 2, 4, 8])), 0, 0), mb=(mb1, 0, 0))
        out.append((layer, variant, tuning))
    return out


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
def test_random_layers_and_tilings_through_the_one_launch_kernels(orc, layout):
    """40 seeded random (layer, variant, tile, wavefronts, stage-1 width) combinations per layout; a combination the
    library refuses (register tile not compiled, tile too large for LDS) is skipped, at least 20 must run."""
    ran = 0
    for layer, variant, tuning in _random_cases(40, 20221103 + layout):
        if layout == B.LAYOUT_NHWC and (layer.C % 4 or layer.N % 4):
            layer = Layer(layer.batch, 4 * ((layer.C + 3) // 4), 4 * ((layer.N + 3) // 4), layer.H, layer.W, layer.R1, layer.R2,
                          layer.K, layer.stride, layer.pad)
        _announce("random", layer.name(), variant, tuning, "layout", layout)
        inputs = make_inputs(layer, 1000 + ran)
        try:
            got, desc = run_gpu_layout(layer, inputs, B.make_tuning(variant=VARIANTS[variant], **tuning), layout)
        except B.TdcError as e:
            assert e.status in (B.TDC_ERR_BAD_TUNING, B.TDC_ERR_UNSUPPORTED), e
            continue
        want = _oracle(orc, layer, inputs)
        if layout == B.LAYOUT_NHWC:
            want = np.ascontiguousarray(np.transpose(want, (0, 2, 3, 1)))
        assert_parity(got, want, desc)
        ran += 1
    assert ran >= 20, ran


def run_gpu_layout(layer, inputs, tuning, layout):
    """One call on cuda:0 in the given activation layout; returns (y as numpy in that layout, plan description)."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    dev = torch.device("cuda:0")
    t = {k: torch.from_numpy(v).to(dev) for k, v in inputs.items()}
    conv = TuckerConv2d(layer, 0, tuning, layout=layout)
    try:
        conv.pack(t["U_in"], t["core"], t["U_out"])
        x = t["x"].permute(0, 2, 3, 1).contiguous() if layout == B.LAYOUT_NHWC else t["x"]
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        conv(x, y)
        torch.cuda.synchronize()
        return y.cpu().numpy(), conv.describe()
    finally:
        conv.close()


def test_error_paths_on_device():
    import ctypes
    import torch
    layer = Layer(1, 8, 8, 6, 6, 4, 4)
    _announce("errors", layer.name())
    lib = B.load()
    s = B.make_shape(**layer.asdict())
    plan = B.tdc_plan_create(s, 0)
    t = {k: torch.from_numpy(v).cuda() for k, v in make_inputs(layer, 1).items()}
    y = torch.empty((1, 8, 6, 6), device="cuda")
    other = B.make_shape(1, 8, 8, 6, 7, 4, 4)
    st = torch.cuda.current_stream().cuda_stream
    args = [t["x"].data_ptr(), t["U_in"].data_ptr(), t["core"].data_ptr(), t["U_out"].data_ptr(), y.data_ptr()]
    assert lib.tdc_conv_tucker2(plan, st, *args, ctypes.byref(other)) == B.TDC_ERR_SHAPE_MISMATCH
    for i in range(5):
        a = list(args)
        a[i] = None
        assert lib.tdc_conv_tucker2(plan, st, *a, ctypes.byref(s)) == B.TDC_ERR_NULL
    assert lib.tdc_conv_tucker2(plan, st, *args, None) == B.TDC_ERR_NULL
    assert lib.tdc_conv_tucker2(plan, st, *args, ctypes.byref(s)) == B.TDC_OK
    assert B.tdc_plan_workspace_bytes(plan) > 0 and B.tdc_plan_kernel_count(plan) in (1, 2, 3)
    p2 = ctypes.c_void_p()
    assert lib.tdc_plan_create(ctypes.byref(p2), ctypes.byref(s), 99) == B.TDC_ERR_HIP
    with pytest.raises(B.TdcError):
        B.tdc_plan_create(s, 0, B.make_tuning(variant=B.VARIANT_FUSED, tile_h=64, tile_w=64))
    torch.cuda.synchronize()
    B.tdc_plan_destroy(plan)
