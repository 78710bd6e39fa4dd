"""GPU parity of tdc_conv_dense (the undecomposed K x K layer, Eq. 1's kernel applied directly)
against the oracle's dense convolution, through the C ABI."""
import ctypes
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.workloads import Layer, config_layers, layer_seed, make_dense_inputs, make_inputs
from parity_util import assert_parity

pytestmark = pytest.mark.gpu


def _announce(*parts):
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def _run(layer, inputs, tuning=None, pack=True):
    import torch
    from paper_2211_03715_amd.layer import DenseConv2d
    dev = torch.device("cuda:0")
    x, W = (torch.from_numpy(inputs[k]).to(dev) for k in ("x", "W"))
    conv = DenseConv2d(layer, 0, tuning)
    try:
        if pack:
            conv.pack(W)
        y = torch.full((layer.batch, layer.N, conv.Ho, conv.Wo), float("nan"), device=dev, dtype=torch.float32)
        conv(x, y, W=W)
        torch.cuda.synchronize()
        return y.cpu().numpy(), conv.describe()
    finally:
        conv.close()


# R1, R2 are ignored by a dense plan; they only have to be positive.
SMALL = [
    Layer(1, 5, 7, 6, 9, 1, 1),                  # nothing a multiple of anything, C < 16
    Layer(2, 20, 24, 19, 23, 3, 3),              # C and N just over a 16-block, odd image
    Layer(3, 33, 18, 12, 40, 8, 8, 3, 2, 1),     # stride 2, batch 3
    Layer(1, 16, 16, 9, 9, 4, 4, 3, 1, 0),       # no padding
    Layer(2, 12, 10, 7, 5, 4, 6, 1, 1, 0),       # 1x1
    Layer(1, 8, 8, 11, 13, 5, 3, 5, 1, 2),       # 5x5
    Layer(1, 3, 2, 1, 1, 1, 1, 1, 1, 0),         # a single pixel
    Layer(1, 64, 64, 56, 56, 16, 16),            # the primary layer's original convolution
    Layer(1, 40, 72, 16, 16, 32, 48, 3, 2, 1),
]


@pytest.mark.parametrize("layer", SMALL, ids=lambda l: l.name())
def test_dense_small_shapes(orc, layer):
    _announce("dense small", layer.name())
    inputs = make_dense_inputs(layer, 4321)
    want, _ = orc.conv_dense_with(orc.Shape(**layer.asdict()), inputs["x"], inputs["W"].astype(np.float64))
    got, desc = _run(layer, inputs)
    e = assert_parity(got, want, "dense %s [%s]" % (layer.name(), desc))
    print("   ", desc, "E_inf=%.2e E_el=%.2e" % e, flush=True)


FORCED = [dict(mb=(0, 1, 0), pb=(0, 1, 0), waves=(0, 1, 0)), dict(mb=(0, 2, 0), pb=(0, 2, 0), waves=(0, 4, 0)),
          dict(mb=(0, 4, 0), pb=(0, 1, 0), waves=(0, 8, 0)), dict(mb=(0, 1, 0), pb=(0, 4, 0), waves=(0, 3, 0)),
          dict(mb=(0, 2, 0), pb=(0, 1, 0), waves=(0, 6, 0))]


@pytest.mark.parametrize("tuning", FORCED, ids=lambda t: "mb%d_pb%d_w%d" % (t["mb"][1], t["pb"][1], t["waves"][1]))
def test_dense_forced_tunings(orc, tuning):
    layer = Layer(2, 40, 64, 19, 23, 1, 1)
    _announce("dense forced", tuning)
    inputs = make_dense_inputs(layer, 99)
    want, _ = orc.conv_dense_with(orc.Shape(**layer.asdict()), inputs["x"], inputs["W"].astype(np.float64))
    got, desc = _run(layer, inputs, B.make_tuning(**tuning))
    assert_parity(got, want, desc)
    got2, _ = _run(layer, inputs, B.make_tuning(**tuning), pack=False)      # re-layout on every call
    assert np.array_equal(got, got2)


def test_dense_full_size_layers_of_the_sweep(orc):
    """The original convolutions of the batch-1 ResNet-18-shaped sweep, at full size."""
    for i, layer in enumerate(config_layers(2)):
        _announce("dense config 2 layer", i, layer.name())
        inputs = make_dense_inputs(layer, layer_seed(2, i) + 500)
        want, _ = orc.conv_dense_with(orc.Shape(**layer.asdict()), inputs["x"], inputs["W"].astype(np.float64))
        got, desc = _run(layer, inputs)
        e = assert_parity(got, want, "dense %s [%s]" % (layer.name(), desc))
        print("   ", desc, "E_inf=%.2e E_el=%.2e" % e, flush=True)


def test_dense_of_reconstructed_kernel_matches_the_tucker_layer(orc):
    """Eq. 1: the dense layer with K = core x1 U_in x2 U_out gives what the Tucker layer gives."""
    import torch
    from parity_util import run_gpu
    layer = Layer(1, 24, 20, 14, 14, 12, 9)
    _announce("dense vs tucker", layer.name())
    inputs = make_inputs(layer, 5)
    sh = orc.Shape(**layer.asdict())
    Wd, _ = orc.reconstruct(sh, inputs["U_in"], inputs["core"], inputs["U_out"])
    got_dense, _ = _run(layer, {"x": inputs["x"], "W": np.ascontiguousarray(Wd.astype(np.float32))})
    got_tucker, _ = run_gpu(layer, inputs, None)
    want, _ = orc.conv_factored(sh, **inputs)
    assert_parity(got_dense, want, "dense of reconstructed kernel")
    assert_parity(got_tucker, want, "tucker")
    torch.cuda.synchronize()


def test_dense_and_tucker_plans_reject_each_others_calls():
    import torch
    layer = Layer(1, 8, 8, 6, 6, 4, 4)
    _announce("dense errors", layer.name())
    lib = B.load()
    s = B.make_shape(**layer.asdict())
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(v).cuda() for k, v in make_inputs(layer, 1).items()}
    W = torch.from_numpy(make_dense_inputs(layer, 1)["W"]).cuda()
    y = torch.empty((1, 8, 6, 6), device="cuda")
    dense = B.tdc_plan_create(s, 0, B.make_tuning(variant=B.VARIANT_DENSE))
    tucker = B.tdc_plan_create(s, 0)
    p = lambda a: a.data_ptr()
    assert lib.tdc_conv_tucker2(dense, st, p(t["x"]), p(t["U_in"]), p(t["core"]), p(t["U_out"]), p(y),
                                ctypes.byref(s)) == B.TDC_ERR_BAD_TUNING
    assert lib.tdc_plan_pack_weights(dense, st, p(t["U_in"]), p(t["core"]), p(t["U_out"])) == B.TDC_ERR_BAD_TUNING
    assert lib.tdc_conv_dense(tucker, st, p(t["x"]), p(W), p(y), ctypes.byref(s)) == B.TDC_ERR_BAD_TUNING
    assert lib.tdc_plan_pack_dense(tucker, st, p(W)) == B.TDC_ERR_BAD_TUNING
    assert lib.tdc_conv_dense(dense, st, None, p(W), p(y), ctypes.byref(s)) == B.TDC_ERR_NULL
    other = B.make_shape(1, 8, 8, 6, 7, 4, 4)
    assert lib.tdc_conv_dense(dense, st, p(t["x"]), p(W), p(y), ctypes.byref(other)) == B.TDC_ERR_SHAPE_MISMATCH
    assert lib.tdc_conv_dense(dense, st, p(t["x"]), p(W), p(y), ctypes.byref(s)) == B.TDC_OK
    assert B.tdc_plan_kernel_count(dense) == 1 and B.tdc_plan_workspace_bytes(dense) > 0
    torch.cuda.synchronize()
    B.tdc_plan_destroy(dense)
    B.tdc_plan_destroy(tucker)


def test_dense_sweep_tool_times_every_tuning_and_names_the_best():
    """autotune --dense: the sweep behind the `dense` coefficient table, on a small layer with a handful of launches."""
    from paper_2211_03715_amd import autotune as A
    layer = Layer(1, 32, 64, 9, 11, 1, 1, 1, 1, 0)
    print("[case] dense sweep tool", layer.name(), flush=True)
    sys.stdout.flush()
    r = A.autotune_dense(layer, iters=5, epilogue="bias_residual_relu", layout=B.LAYOUT_NHWC)
    assert r["layout"] == "nhwc" and r["epilogue"] == "bias_residual_relu" and r["layer"] == layer.name()
    assert len(r["rows"]) >= 12 and all(row["tuning"]["variant"] == "dense" and row["us"] > 0 for row in r["rows"])
    assert r["best"]["us"] == min(row["us"] for row in r["rows"]) and r["auto"]["us"] > 0
    # what the fit reads back: the dense model's terms for every timed tuning
    shape = B.make_shape(**layer.asdict(), layout=B.LAYOUT_NHWC)
    t = r["best"]["tuning"]
    model, names, terms = B.tdc_model_terms(shape, B.make_tuning(variant=B.VARIANT_DENSE, waves=tuple(t["waves"]), mb=tuple(t["mb"]), pb=tuple(t["pb"])))
    assert model == "dense" and names[-2:] == ["y_nchw", "y_nhwc"] and terms[-2] == 0.0 and terms[-1] > 0.0
