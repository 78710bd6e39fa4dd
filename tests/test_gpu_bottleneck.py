"""A bottleneck block (dense 1x1 + Tucker 3x3 + dense 1x1, epilogues fused) against the oracle, eagerly
and replayed from a HIP graph."""
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.bottleneck import TuckerBottleneck, make_block_weights
from parity_util import assert_parity

pytestmark = pytest.mark.gpu


def _oracle_block(orc, blk, w, x):
    y1, _ = orc.conv_dense_with(orc.Shape(**blk.l1.asdict()), x, w["W1"].astype(np.float64))
    t1 = orc.apply_epilogue(y1, w["b1"], None, True).astype(np.float32)        # the GPU stores t1, t2 in fp32
    y2, _ = orc.conv_factored(orc.Shape(**blk.l2.asdict()), t1, w["U_in"], w["core"], w["U_out"])
    t2 = orc.apply_epilogue(y2, w["b2"], None, True).astype(np.float32)
    y3, _ = orc.conv_dense_with(orc.Shape(**blk.l3.asdict()), t2, w["W3"].astype(np.float64))
    return orc.apply_epilogue(y3, w["b3"], x, True)


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("shape", [(1, 64, 16, 14, 14, 8, 8), (2, 48, 24, 9, 11, 16, 20), (1, 256, 64, 56, 56, 16, 16)],
                         ids=lambda s: "b%d_c%d_m%d_%dx%d_r%d-%d" % s)
def test_bottleneck_eager_and_graph(orc, shape, layout):
    import torch
    batch, C, M, H, W, R1, R2 = shape
    print("[case] bottleneck", shape, "layout", layout, flush=True)
    sys.stdout.flush()
    w = make_block_weights(C, M, R1, R2, 11)
    blk = TuckerBottleneck(batch, C, M, H, W, R1, R2, w, layout=layout)
    perm = (lambda a: np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))) if layout == B.LAYOUT_NHWC else (lambda a: a)
    try:
        rng = np.random.default_rng(5)
        xs = [rng.standard_normal((batch, C, H, W), dtype=np.float32) for _ in range(3)]
        wants = [perm(_oracle_block(orc, blk, w, x)) for x in xs]       # the oracle works in NCHW
        xs = [perm(x) for x in xs]
        x_dev = torch.from_numpy(xs[0]).to(blk.dev)
        got = blk(x_dev)
        torch.cuda.synchronize()
        assert_parity(got.cpu().numpy(), wants[0], "eager " + blk.describe())
        # graph: captured once, replayed on new inputs, with eager work and synchronisations in between
        x_static = torch.empty_like(x_dev)
        graph = blk.capture(x_static)
        for rep in range(2):
            for x, want in zip(xs, wants):
                x_static.copy_(torch.from_numpy(x).to(blk.dev))
                blk.y.fill_(float("nan"))
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert_parity(blk.y.cpu().numpy(), want, "graph replay")
                eager = blk(x_static).clone()                 # the same block, eagerly, between replays
                torch.cuda.synchronize()
                assert torch.equal(eager, blk.y)
                assert_parity(eager.cpu().numpy(), want, "eager between replays")
    finally:
        blk.close()


@pytest.mark.parametrize("variant", [B.VARIANT_FUSED, B.VARIANT_CHAIN], ids=["fused", "chain"])
def test_large_lds_kernels_under_graph_capture(orc, variant):
    """The throughput kernels ask for more dynamic LDS than the default limit; that request must not disturb
    a capture (it is made before the first launch and remembered), and every replay must match the oracle."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    from paper_2211_03715_amd.workloads import Layer, make_inputs
    layer = Layer(8, 128, 128, 28, 28, 32, 32)
    print("[case] graph capture, large LDS", layer.name(), variant, flush=True)
    sys.stdout.flush()
    dev = torch.device("cuda:0")
    sets = [make_inputs(layer, seed) for seed in (31, 32)]
    sets[1] = dict(sets[0], x=sets[1]["x"])          # one set of weights (the packed one), two inputs
    wants = [orc.conv_factored(orc.Shape(**layer.asdict()), **inp)[0] for inp in sets]
    t = {k: torch.from_numpy(v).to(dev) for k, v in sets[0].items()}
    conv = TuckerConv2d(layer, 0, B.make_tuning(variant=variant, tile_h=4, tile_w=28, waves=(4, 4, 4), mb=(1, 1, 1),
                                              pb=(1, 1, 1)))   # two groups of pixel blocks per wavefront: the chain kernel stages its weights in LDS
    try:
        assert "lds=" in conv.describe() and int(conv.describe().split("lds=")[1].split("B")[0]) > 48 * 1024
        conv.pack(t["U_in"], t["core"], t["U_out"])
        x_static = torch.empty_like(t["x"])
        y = torch.full(conv.out_shape(), float("nan"), device=dev)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):          # the very first launch of this plan is the captured one
            conv.bind(x_static, y)()
        for rep in range(3):
            for inp, want in zip(sets, wants):
                x_static.copy_(torch.from_numpy(inp["x"]).to(dev))
                y.fill_(float("nan"))
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert_parity(y.cpu().numpy(), want, "replay %d [%s]" % (rep, conv.describe()))
                eager = conv(x_static)
                torch.cuda.synchronize()
                assert torch.equal(eager, y)
    finally:
        conv.close()
