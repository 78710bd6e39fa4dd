"""A bottleneck block (dense 1x1 + Tucker 3x3 + dense 1x1, epilogues fused) against the oracle, eagerly
and replayed from a HIP graph; blocks with stride 2 and a projection shortcut; and the 3 + 4 + 6 + 3 blocks of a
ResNet-50-shaped network chained, eagerly and as one graph."""
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.bottleneck import TuckerBottleneck, TuckerResNetBody, make_block_weights
from parity_util import assert_parity

pytestmark = pytest.mark.gpu


def _oracle_block(orc, blk, w, x):
    y1, _ = orc.conv_dense_with(orc.Shape(**blk.l1.asdict()), x, w["W1"].astype(np.float64))
    t1 = orc.apply_epilogue(y1, w["b1"], None, True).astype(np.float32)        # the GPU stores t1, t2 in fp32
    y2, _ = orc.conv_factored(orc.Shape(**blk.l2.asdict()), t1, w["U_in"], w["core"], w["U_out"])
    t2 = orc.apply_epilogue(y2, w["b2"], None, True).astype(np.float32)
    y3, _ = orc.conv_dense_with(orc.Shape(**blk.l3.asdict()), t2, w["W3"].astype(np.float64))
    s = x
    if blk.projection:                                                          # s = Wp (*) x + bp, stored in fp32
        yp, _ = orc.conv_dense_with(orc.Shape(**blk.lp.asdict()), x, w["Wp"].astype(np.float64))
        s = orc.apply_epilogue(yp, w["bp"], None, False).astype(np.float32)
    return orc.apply_epilogue(y3, w["b3"], s, True)


def _perm(layout):
    return (lambda a: np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))) if layout == B.LAYOUT_NHWC else (lambda a: a)


def _unperm(layout):
    return (lambda a: np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))) if layout == B.LAYOUT_NHWC else (lambda a: a)


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
    perm = _perm(layout)
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


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("shape", [(1, 32, 16, 14, 14, 8, 8, 2, 64), (2, 24, 12, 9, 11, 8, 12, 2, 48), (1, 16, 16, 10, 7, 8, 8, 1, 64),
                                   (1, 256, 128, 56, 56, 32, 32, 2, 512)],
                         ids=lambda s: "b%d_c%d_m%d_%dx%d_r%d-%d_s%d_out%d" % s)
def test_projection_block(orc, shape, layout):
    """The first block of a stage: stride on the 3x3 convolution, shortcut through a strided 1x1 projection."""
    import torch
    batch, C, M, H, W, R1, R2, stride, C_out = shape
    print("[case] projection block", shape, "layout", layout, flush=True)
    sys.stdout.flush()
    w = make_block_weights(C, M, R1, R2, 13, C_out=C_out, projection=True)
    blk = TuckerBottleneck(batch, C, M, H, W, R1, R2, w, layout=layout, stride=stride, C_out=C_out)
    perm = _perm(layout)
    try:
        assert blk.projection and blk.kernels() >= 4
        rng = np.random.default_rng(6)
        xs = [rng.standard_normal((batch, C, H, W), dtype=np.float32) for _ in range(2)]
        wants = [perm(_oracle_block(orc, blk, w, x)) for x in xs]
        x_static = torch.from_numpy(perm(xs[0])).to(blk.dev)
        got = blk(x_static)
        torch.cuda.synchronize()
        assert tuple(got.shape) == wants[0].shape
        assert_parity(got.cpu().numpy(), wants[0], "eager " + blk.describe())
        graph = blk.capture(x_static)
        for x, want in zip(xs[::-1], wants[::-1]):
            x_static.copy_(torch.from_numpy(perm(x)).to(blk.dev))
            blk.y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert_parity(blk.y.cpu().numpy(), want, "graph replay")
    finally:
        blk.close()


def _oracle_network(orc, net, x):
    """The oracle chained block by block; every tensor the GPU stores (block outputs included) is rounded to fp32."""
    outs = []
    for blk, w in zip(net.blocks, net.weights):
        x = _oracle_block(orc, blk, w, x).astype(np.float32)
        outs.append(x)
    return outs


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("case", [(2, 16, 32, 32), (1, 64, 56, 56)], ids=["b2_width16_32x32", "resnet50_b1_width64_56x56"])
def test_resnet_body_eager_and_one_graph(orc, case, layout):
    """3 + 4 + 6 + 3 bottleneck blocks (projection + stride 2 where a stage starts) run back to back.  Compared with
    the oracle chained through all 16 blocks (whole-network parity, the tolerance of a single layer), and block by
    block on the input the GPU itself produced; then the whole network replayed from ONE HIP graph on new inputs."""
    import torch
    batch, width, H, W = case
    print("[case] resnet body", case, "layout", layout, flush=True)
    sys.stdout.flush()
    net = TuckerResNetBody(batch, H, W, width, layout=layout, seed=40)
    perm, unperm = _perm(layout), _unperm(layout)
    try:
        assert len(net.blocks) == 16 and [b.projection for b in net.blocks] == [i in (0, 3, 7, 13) for i in range(16)]
        assert [b.l2.stride for b in net.blocks] == [2 if i in (3, 7, 13) else 1 for i in range(16)]
        rng = np.random.default_rng(8)
        xs = [rng.standard_normal((batch, width, H, W), dtype=np.float32) for _ in range(2)]
        x_static = torch.from_numpy(perm(xs[0])).to(net.dev)
        got = net(x_static)
        torch.cuda.synchronize()
        assert tuple(got.shape) == ((batch, H // 8, W // 8, 32 * width) if layout == B.LAYOUT_NHWC else (batch, 32 * width, H // 8, W // 8))
        wants = _oracle_network(orc, net, xs[0])
        for i, (blk, want) in enumerate(zip(net.blocks, wants)):
            assert_parity(blk.y.cpu().numpy(), perm(want), "network up to block %d" % i)
        # block by block on the GPU's own block inputs: an error in one block cannot hide behind the others
        x_in = xs[0]
        for i, (blk, w) in enumerate(zip(net.blocks, net.weights)):
            assert_parity(blk.y.cpu().numpy(), perm(_oracle_block(orc, blk, w, x_in)), "block %d alone" % i)
            x_in = unperm(blk.y.cpu().numpy())
        eager_first = got.clone()
        graph = net.capture(x_static)
        n_kernels = net.kernels()
        assert n_kernels >= 16 * 3 + 4
        for rep, k in enumerate((1, 0, 1)):
            x_static.copy_(torch.from_numpy(perm(xs[k])).to(net.dev))
            for blk in net.blocks:
                blk.y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            replayed = net.y.clone()
            if k == 0:
                assert torch.equal(replayed, eager_first)
            else:
                assert_parity(replayed.cpu().numpy(), perm(_oracle_network(orc, net, xs[1])[-1]), "graph replay %d" % rep)
            eager = net(x_static).clone()                     # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(eager, replayed)
    finally:
        net.close()


def _oracle_basic_block(orc, blk, w, x):
    ya, _ = orc.conv_factored(orc.Shape(**blk.la.asdict()), x, w["Ua_in"], w["core_a"], w["Ua_out"])
    t1 = orc.apply_epilogue(ya, w["b1"], None, True).astype(np.float32)        # the GPU stores t1 in fp32
    yb, _ = orc.conv_factored(orc.Shape(**blk.lb.asdict()), t1, w["Ub_in"], w["core_b"], w["Ub_out"])
    s = x
    if blk.projection:
        yp, _ = orc.conv_dense_with(orc.Shape(**blk.lp.asdict()), x, w["Wp"].astype(np.float64))
        s = orc.apply_epilogue(yp, w["bp"], None, False).astype(np.float32)
    return orc.apply_epilogue(yb, w["b2"], s, True)


@pytest.mark.parametrize("layout", [B.LAYOUT_NCHW, B.LAYOUT_NHWC], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("case", [(2, 16, 32, 32), (1, 64, 56, 56)], ids=["b2_width16_32x32", "resnet18_b1_width64_56x56"])
def test_resnet18_body_eager_and_one_graph(orc, case, layout):
    """2 + 2 + 2 + 2 basic blocks, both 3x3 convolutions of each in Tucker-2 form (16 Tucker layers: at full size the
    shapes of the batch-1 benchmark sweep and its stride-2 layers, chained with their shortcuts).  Every block's output
    against the oracle chained from the network input, every block alone on the input the GPU gave it, and the whole
    network replayed from ONE HIP graph on changing inputs with eager runs in between."""
    import torch
    from paper_2211_03715_amd.bottleneck import TuckerResNet18Body
    batch, width, H, W = case
    print("[case] resnet18 body", case, "layout", layout, flush=True)
    sys.stdout.flush()
    net = TuckerResNet18Body(batch, H, W, width, layout=layout, seed=60)
    perm, unperm = _perm(layout), _unperm(layout)

    def oracle_network(x):
        outs = []
        for blk, w in zip(net.blocks, net.weights):
            x = _oracle_basic_block(orc, blk, w, x).astype(np.float32)
            outs.append(x)
        return outs

    try:
        assert len(net.blocks) == 8 and [b.projection for b in net.blocks] == [i in (2, 4, 6) for i in range(8)]
        assert [b.la.stride for b in net.blocks] == [2 if i in (2, 4, 6) else 1 for i in range(8)]
        assert [(b.la.R1, b.la.R2) for b in net.blocks[:3]] == [(width // 4, width // 4)] * 2 + [(width // 4, width // 2)]
        rng = np.random.default_rng(9)
        xs = [rng.standard_normal((batch, width, H, W), dtype=np.float32) for _ in range(2)]
        x_static = torch.from_numpy(perm(xs[0])).to(net.dev)
        got = net(x_static)
        torch.cuda.synchronize()
        assert tuple(got.shape) == ((batch, H // 8, W // 8, 8 * width) if layout == B.LAYOUT_NHWC else (batch, 8 * width, H // 8, W // 8))
        wants = oracle_network(xs[0])
        for i, (blk, want) in enumerate(zip(net.blocks, wants)):
            assert_parity(blk.y.cpu().numpy(), perm(want), "network up to block %d" % i)
        x_in = xs[0]
        for i, (blk, w) in enumerate(zip(net.blocks, net.weights)):
            assert_parity(blk.y.cpu().numpy(), perm(_oracle_basic_block(orc, blk, w, x_in)), "block %d alone" % i)
            x_in = unperm(blk.y.cpu().numpy())
        eager_first = got.clone()
        graph = net.capture(x_static)
        assert net.kernels() >= 16 + 3
        for rep, k in enumerate((1, 0, 1)):
            x_static.copy_(torch.from_numpy(perm(xs[k])).to(net.dev))
            for blk in net.blocks:
                blk.y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            replayed = net.y.clone()
            if k == 0:
                assert torch.equal(replayed, eager_first)
            else:
                assert_parity(replayed.cpu().numpy(), perm(oracle_network(xs[1])[-1]), "graph replay %d" % rep)
            eager = net(x_static).clone()
            torch.cuda.synchronize()
            assert torch.equal(eager, replayed)
    finally:
        net.close()


def test_blocks_take_tunings_per_convolution(orc):
    """The ``tunings`` hook of the blocks (what bottleneck.oracle_tunings plugs into): every convolution gets the tuning the
    function returns for its kind, layer and epilogue, and the block still matches the oracle."""
    import torch
    from paper_2211_03715_amd.bottleneck import TuckerBasicBlock, make_basic_weights
    print("[case] blocks with given tunings", flush=True)
    sys.stdout.flush()
    asked = []

    def tunings(kind, layer, epilogue):
        asked.append((kind, layer.name(), epilogue))
        if kind == "dense":
            return B.make_tuning(mb=(0, 1, 0), pb=(0, 2, 0), waves=(0, 2, 0))
        return B.make_tuning(variant=B.VARIANT_SPLIT, waves=(2, 2, 2), mb=(1, 1, 1), pb=(1, 1, 1))

    w = make_block_weights(32, 16, 8, 8, 3, C_out=64, projection=True)
    blk = TuckerBottleneck(2, 32, 16, 14, 14, 8, 8, w, stride=2, C_out=64, tunings=tunings)
    try:
        assert [a[0] for a in asked] == ["dense", "tucker", "dense", "dense"] and asked[2][2] == (True, True, True)
        assert "split" in blk.conv2.describe() and "(mb,pb,waves)=(1,2,2)" in blk.conv1.describe()
        x = np.random.default_rng(4).standard_normal((2, 32, 14, 14), dtype=np.float32)
        got = blk(torch.from_numpy(x).to(blk.dev))
        torch.cuda.synchronize()
        assert_parity(got.cpu().numpy(), _oracle_block(orc, blk, w, x), blk.describe())
    finally:
        blk.close()
    wb = make_basic_weights(16, 32, (8, 8), (8, 8), 5, projection=True)
    bb = TuckerBasicBlock(1, 16, 32, 12, 12, (8, 8), (8, 8), wb, stride=2, tunings=tunings)
    try:
        assert "split" in bb.conva.describe() and "split" in bb.convb.describe()
        x = np.random.default_rng(6).standard_normal((1, 16, 12, 12), dtype=np.float32)
        got = bb(torch.from_numpy(x).to(bb.dev))
        torch.cuda.synchronize()
        assert_parity(got.cpu().numpy(), _oracle_basic_block(orc, bb, wb, x), bb.describe())
    finally:
        bb.close()
