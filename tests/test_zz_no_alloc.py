"""The entry point that allocates nothing, tdc_conv_tucker2_static, through the C ABI.

It must give what tdc_conv_tucker2 gives on a SPLIT plan (the existing entry point whose kernels use the
scratch memory that here lives in a static device array): on two calls in a row, the second on a smaller
layer, so that whatever the first left in the shared array would show.  The oracle is checked as well.
Collected last on purpose (see the file name): the round's GPU run stops at the first failure.
"""
import ctypes
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


def _setup(layer, seed, layout):
    import torch
    dev = torch.device("cuda:0")
    inp = make_inputs(layer, seed)
    t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
    if layout == B.LAYOUT_NHWC:
        t["x"] = t["x"].permute(0, 2, 3, 1).contiguous()
    shape = B.make_shape(**layer.asdict(), layout=layout)
    yshape = (layer.batch, layer.Ho, layer.Wo, layer.N) if layout == B.LAYOUT_NHWC else (layer.batch, layer.N, layer.Ho, layer.Wo)
    return inp, t, shape, yshape


def _args(t, y):
    return [ctypes.c_void_p(a.data_ptr()) for a in (t["x"], t["U_in"], t["core"], t["U_out"], y)]


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
def test_static_entry_point_twice_second_smaller(orc, layout):
    import torch
    lib = B.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    big = Layer(3, 36, 44, 21, 26, 20, 28, 3, 1, 1)
    small = Layer(1, 12, 20, 9, 11, 5, 7, 3, 2, 1)       # fewer of everything: stale scratch would be in reach
    cases = [(L, _setup(L, seed, layout)) for L, seed in ((big, 41), (small, 42))]
    # the two calls in a row, nothing between them
    got = []
    for L, (inp, t, shape, yshape) in cases:
        _announce("static", "nhwc" if layout else "nchw", L.name())
        y = torch.full(yshape, float("nan"), device=dev, dtype=torch.float32)
        rc = lib.tdc_conv_tucker2_static(stream, *_args(t, y), ctypes.byref(shape))
        assert rc == B.TDC_OK, B.status_string(rc)
        got.append(y)
    torch.cuda.synchronize()
    for (L, (inp, t, shape, yshape)), y_static in zip(cases, got):
        _announce("split plan", "nhwc" if layout else "nchw", L.name())
        plan = ctypes.c_void_p()
        forced = B.make_tuning(variant=B.VARIANT_SPLIT)
        assert lib.tdc_plan_create_tuned(ctypes.byref(plan), ctypes.byref(shape), 0, ctypes.byref(forced)) == B.TDC_OK
        try:
            y_plan = torch.full(yshape, float("nan"), device=dev, dtype=torch.float32)
            x, u1, co, u2, yp = _args(t, y_plan)
            rc = lib.tdc_conv_tucker2(plan, stream, x, u1, co, u2, yp, ctypes.byref(shape))
            assert rc == B.TDC_OK, B.status_string(rc)
            torch.cuda.synchronize()
        finally:
            lib.tdc_plan_destroy(plan)
        a, b = y_static.cpu().numpy(), y_plan.cpu().numpy()
        if layout == B.LAYOUT_NHWC:
            a, b = np.transpose(a, (0, 3, 1, 2)), np.transpose(b, (0, 3, 1, 2))
        assert np.isfinite(a).all()
        assert_parity(a, b, "static vs SPLIT plan %s" % L.name())
        assert np.array_equal(a, b), "same kernels, same tuning: the two entry points must agree bit for bit"
        want, _ = orc.conv_factored(orc.Shape(**L.asdict()), **inp)
        assert_parity(a, want, "static vs oracle %s" % L.name())


def test_static_entry_point_rejects_what_does_not_fit():
    import torch
    lib = B.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # z1 alone: 64 * 16 * 512 * 512 floats = 1 GiB > the 32 MiB array.  Nothing is enqueued, so the (small)
    # buffers passed are never touched.
    shape = B.make_shape(64, 16, 16, 512, 512, 16, 16)
    buf = torch.zeros(1024, device=dev)
    p = ctypes.c_void_p(buf.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert lib.tdc_conv_tucker2_static(stream, p, p, p, p, p, ctypes.byref(shape)) == B.TDC_ERR_TOO_LARGE
    assert "static" in B.status_string(B.TDC_ERR_TOO_LARGE)
    assert lib.tdc_conv_tucker2_static(stream, None, p, p, p, p, ctypes.byref(shape)) == B.TDC_ERR_NULL
    bad = B.make_shape(1, 16, 16, 8, 8, 4, 4, 9, 1, 1)
    assert lib.tdc_conv_tucker2_static(stream, p, p, p, p, p, ctypes.byref(bad)) == B.TDC_ERR_UNSUPPORTED
    torch.cuda.synchronize()
