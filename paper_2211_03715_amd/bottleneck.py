"""A ResNet bottleneck block whose 3x3 convolution is in Tucker-2 form, on this library.

The paper's end-to-end models (section 7.3) keep the 1x1 convolutions of a bottleneck dense and
replace the 3x3 one by the Tucker-2 layer; batch-norm is folded into weights and bias at
inference.  One block is three calls, each with its epilogue fused into the store of its output:

    t1 = relu(W1 (*) x  + b1)                  1x1, C -> M            tdc_conv_dense_ex
    t2 = relu(Tucker3x3(t1) + b2)              M -> R1 -> R2 -> M     tdc_conv_tucker2_ex
    y  = relu(W3 (*) t2 + b3 + x)              1x1, M -> C, shortcut  tdc_conv_dense_ex

All buffers are allocated when the block is built, so a call only enqueues three launches
(four when the selector gives the Tucker layer two kernels) and can be captured into a HIP
graph: `graph = block.capture(x_static)`, then `graph.replay()`.

A block that changes width or resolution (the first of a ResNet stage) has stride 2 on its 3x3 convolution and
a projection shortcut, one more dense 1x1 launch:   s = Wp (*) x + bp,   y = relu(W3 (*) t2 + b3 + s).
TuckerResNetBody strings 3 + 4 + 6 + 3 such blocks into the residual stages of a ResNet-50-shaped network.

TuckerBasicBlock is the two-convolution block of the shallower networks, both 3x3 convolutions in Tucker-2 form:
    t1 = relu(Tucker3x3_a(x) + b1)             C -> M, stride s
    y  = relu(Tucker3x3_b(t1) + b2 + s(x))     M -> M; s(x) = x, or Wp (*) x + bp where the block changes shape
and TuckerResNet18Body the 2 + 2 + 2 + 2 of them of a ResNet-18-shaped network (16 Tucker layers: the shapes of the
batch-1 benchmark sweep, in sequence, with their shortcuts and epilogues).

    python -m paper_2211_03715_amd.bottleneck [--nhwc]             # eager vs graph latency of a few block shapes
    python -m paper_2211_03715_amd.bottleneck --resnet50 [--nhwc] [--batch B]   # the 16-block network
    python -m paper_2211_03715_amd.bottleneck --resnet18 [--nhwc] [--batch B]   # the 8 basic blocks
    ... --oracle    # then once more with every convolution's tuning found by exhaustive search (minutes)
"""
from __future__ import annotations

import sys
from typing import Dict

import numpy as np

from . import binding as B
from .layer import DenseConv2d, TuckerConv2d
from .workloads import Layer


def make_block_weights(C: int, M: int, R1: int, R2: int, seed: int, C_out: int = 0, projection: bool = False) -> Dict[str, np.ndarray]:
    """Seeded float32 weights of one block, N(0, 1/fan_in); biases N(0, 0.01).  C_out (default C) is the width the
    block leaves with; with ``projection`` the shortcut is a 1x1 convolution C -> C_out ("Wp", "bp")."""
    rng = np.random.default_rng(seed)
    C_out = C_out or C
    n = lambda shape, fan: (rng.standard_normal(shape, dtype=np.float32) * np.float32(fan ** -0.5))
    w = {"W1": n((C, M, 1, 1), C), "b1": n((M,), 100.0),
         "U_in": n((M, R1), M), "core": n((R1, R2, 3, 3), R1 * 9), "U_out": n((R2, M), R2), "b2": n((M,), 100.0),
         "W3": n((M, C_out, 1, 1), M), "b3": n((C_out,), 100.0)}
    if projection:
        w["Wp"], w["bp"] = n((C, C_out, 1, 1), C), n((C_out,), 100.0)
    return w


class TuckerBottleneck:
    def __init__(self, batch: int, C: int, M: int, H: int, W: int, R1: int, R2: int, weights: Dict, device: int = 0,
                 layout: int = B.LAYOUT_NCHW, stride: int = 1, C_out: int = 0, tunings=None):
        """``layout``: LAYOUT_NCHW (x, y [batch][C][H][W]) or LAYOUT_NHWC ([batch][H][W][C]); C, M multiples of 4 for NHWC.
        ``stride`` sits on the 3x3 convolution; with stride != 1 or C_out != C the shortcut is the projection
        s = Wp (*) x + bp (1x1, same stride, no activation: weights "Wp", "bp") and y = relu(W3 (*) t2 + b3 + s).
        ``tunings``: a function (kind, layer, epilogue) -> tdc_tuning or None that overrides the selector per
        convolution (see oracle_tunings); kind is "dense" or "tucker", epilogue a (bias, residual, relu) triple of bools."""
        import torch
        self.dev = torch.device("cuda", device)
        self.layout = layout
        C_out = C_out or C
        self.projection = stride != 1 or C_out != C
        self.l1 = Layer(batch, C, M, H, W, 1, 1, 1, 1, 0)
        self.l2 = Layer(batch, M, M, H, W, R1, R2, 3, stride, 1)
        self.l3 = Layer(batch, M, C_out, self.l2.Ho, self.l2.Wo, 1, 1, 1, 1, 0)
        self.lp = Layer(batch, C, C_out, H, W, 1, 1, 1, stride, 0) if self.projection else None
        self.w = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.dev) for k, v in weights.items()}
        pick = tunings or (lambda kind, layer, epilogue: None)
        self.conv1 = DenseConv2d(self.l1, device, pick("dense", self.l1, (True, False, True)), layout=layout)
        self.conv2 = TuckerConv2d(self.l2, device, pick("tucker", self.l2, (True, False, True)), layout=layout)
        self.conv3 = DenseConv2d(self.l3, device, pick("dense", self.l3, (True, True, True)), layout=layout)
        self.convp = DenseConv2d(self.lp, device, pick("dense", self.lp, (True, False, False)), layout=layout) if self.projection else None
        self.conv1.pack(self.w["W1"])
        self.conv2.pack(self.w["U_in"], self.w["core"], self.w["U_out"])
        self.conv3.pack(self.w["W3"])
        self.t1 = torch.empty(self.conv1.out_shape(), device=self.dev, dtype=torch.float32)
        self.t2 = torch.empty(self.conv2.out_shape(), device=self.dev, dtype=torch.float32)
        self.y = torch.empty(self.conv3.out_shape(), device=self.dev, dtype=torch.float32)
        self.s = None
        if self.projection:
            self.convp.pack(self.w["Wp"])
            self.s = torch.empty(self.convp.out_shape(), device=self.dev, dtype=torch.float32)
            assert tuple(self.s.shape) == tuple(self.y.shape)
        self._launchers = None
        self._x = None

    def _convs(self):
        return [c for c in (self.convp, self.conv1, self.conv2, self.conv3) if c is not None]

    def bind(self, x):
        """Marshal the block's calls for a fixed input tensor; returns self for chaining."""
        self._x = x
        first = (self.convp.bind(x, self.s, bias=self.w["bp"]),) if self.projection else ()    # while x is the freshest data
        self._launchers = first + (
            self.conv1.bind(x, self.t1, bias=self.w["b1"], relu=True),
            self.conv2.bind(self.t1, self.t2, bias=self.w["b2"], relu=True),
            self.conv3.bind(self.t2, self.y, bias=self.w["b3"], residual=self.s if self.projection else x, relu=True),
        )
        return self

    def __call__(self, x=None):
        """Enqueue the block on the current stream; returns the (block-owned) output tensor."""
        if x is None:
            x = self._x
        if self._launchers is None or x.data_ptr() != self._x.data_ptr():
            self.bind(x)
        for launch in self._launchers:
            launch()
        return self.y

    def capture(self, x_static):
        """Capture the block's launches on x_static into a HIP graph (torch.cuda.CUDAGraph)."""
        import torch
        self.bind(x_static)
        self()                               # once eagerly: kernel attributes, lazy module load
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.bind(x_static)              # launchers carry their stream: bind to the capturing one
            self()
        self._launchers = None               # the next eager call binds to its own current stream
        return graph

    def kernels(self) -> int:
        return 2 + self.conv2.kernel_count() + (1 if self.projection else 0)

    def flops(self) -> int:
        """Algorithmic FLOPs of the block as built (2 per multiply-add; the Tucker layer in its factored form)."""
        from . import roofline as R
        dense = lambda L: 2 * L.batch * L.C * L.N * L.K * L.K * L.Ho * L.Wo
        return dense(self.l1) + R.flops(self.l2) + dense(self.l3) + (dense(self.lp) if self.projection else 0)

    def describe(self) -> str:
        head = "shortcut 1x1: %s | " % self.convp.describe() if self.projection else ""
        return head + "1x1: %s | 3x3: %s | 1x1: %s" % (self.conv1.describe(), self.conv2.describe(), self.conv3.describe())

    def close(self) -> None:
        for c in self._convs():
            c.close()


def make_basic_weights(C: int, M: int, Ra: tuple, Rb: tuple, seed: int, projection: bool = False) -> Dict[str, np.ndarray]:
    """Seeded float32 weights of one basic block, N(0, 1/fan_in); biases N(0, 0.01).  Ra, Rb = (R1, R2) of the two layers."""
    rng = np.random.default_rng(seed)
    n = lambda shape, fan: (rng.standard_normal(shape, dtype=np.float32) * np.float32(fan ** -0.5))
    w = {"Ua_in": n((C, Ra[0]), C), "core_a": n((Ra[0], Ra[1], 3, 3), Ra[0] * 9), "Ua_out": n((Ra[1], M), Ra[1]), "b1": n((M,), 100.0),
         "Ub_in": n((M, Rb[0]), M), "core_b": n((Rb[0], Rb[1], 3, 3), Rb[0] * 9), "Ub_out": n((Rb[1], M), Rb[1]), "b2": n((M,), 100.0)}
    if projection:
        w["Wp"], w["bp"] = n((C, M, 1, 1), C), n((M,), 100.0)
    return w


class TuckerBasicBlock:
    def __init__(self, batch: int, C: int, M: int, H: int, W: int, Ra: tuple, Rb: tuple, weights: Dict, device: int = 0,
                 layout: int = B.LAYOUT_NCHW, stride: int = 1, tunings=None):
        """Two Tucker-2 3x3 convolutions, C -> M (``stride``) and M -> M, ranks Ra = (R1, R2) and Rb; a projection
        shortcut (dense 1x1, same stride, weights "Wp", "bp") when stride != 1 or M != C."""
        import torch
        self.dev = torch.device("cuda", device)
        self.layout = layout
        self.projection = stride != 1 or M != C
        self.la = Layer(batch, C, M, H, W, Ra[0], Ra[1], 3, stride, 1)
        self.lb = Layer(batch, M, M, self.la.Ho, self.la.Wo, Rb[0], Rb[1], 3, 1, 1)
        self.lp = Layer(batch, C, M, H, W, 1, 1, 1, stride, 0) if self.projection else None
        self.w = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.dev) for k, v in weights.items()}
        pick = tunings or (lambda kind, layer, epilogue: None)
        self.conva = TuckerConv2d(self.la, device, pick("tucker", self.la, (True, False, True)), layout=layout)
        self.convb = TuckerConv2d(self.lb, device, pick("tucker", self.lb, (True, True, True)), layout=layout)
        self.convp = DenseConv2d(self.lp, device, pick("dense", self.lp, (True, False, False)), layout=layout) if self.projection else None
        self.conva.pack(self.w["Ua_in"], self.w["core_a"], self.w["Ua_out"])
        self.convb.pack(self.w["Ub_in"], self.w["core_b"], self.w["Ub_out"])
        self.t1 = torch.empty(self.conva.out_shape(), device=self.dev, dtype=torch.float32)
        self.y = torch.empty(self.convb.out_shape(), device=self.dev, dtype=torch.float32)
        self.s = None
        if self.projection:
            self.convp.pack(self.w["Wp"])
            self.s = torch.empty(self.convp.out_shape(), device=self.dev, dtype=torch.float32)
            assert tuple(self.s.shape) == tuple(self.y.shape)
        self._launchers = None
        self._x = None

    def bind(self, x):
        self._x = x
        first = (self.convp.bind(x, self.s, bias=self.w["bp"]),) if self.projection else ()
        wa = (self.w["Ua_in"], self.w["core_a"], self.w["Ua_out"])
        wb = (self.w["Ub_in"], self.w["core_b"], self.w["Ub_out"])
        self._launchers = first + (
            self.conva.bind(x, self.t1, weights=wa, bias=self.w["b1"], relu=True),
            self.convb.bind(self.t1, self.y, weights=wb, bias=self.w["b2"], residual=self.s if self.projection else x, relu=True),
        )
        return self

    def __call__(self, x=None):
        if x is None:
            x = self._x
        if self._launchers is None or x.data_ptr() != self._x.data_ptr():
            self.bind(x)
        for launch in self._launchers:
            launch()
        return self.y

    def kernels(self) -> int:
        return self.conva.kernel_count() + self.convb.kernel_count() + (1 if self.projection else 0)

    def flops(self) -> int:
        from . import roofline as R
        dense = lambda L: 2 * L.batch * L.C * L.N * L.K * L.K * L.Ho * L.Wo
        return R.flops(self.la) + R.flops(self.lb) + (dense(self.lp) if self.projection else 0)

    def describe(self) -> str:
        head = "shortcut 1x1: %s | " % self.convp.describe() if self.projection else ""
        return head + "3x3: %s | 3x3: %s" % (self.conva.describe(), self.convb.describe())

    def close(self) -> None:
        for c in (self.conva, self.convb, self.convp):
            if c is not None:
                c.close()


def default_rank(M: int) -> int:
    """The rank the synthetic networks give a 3x3 layer of M channels: 0.3 M rounded to a multiple of 8, at least 8."""
    return max(8, int(round(0.3 * M / 8.0)) * 8)


class TuckerResNetBody:
    """The four residual stages of a ResNet-50-shaped network (section 7.3's end-to-end setting) with every 3x3 convolution
    in Tucker-2 form: ``blocks`` = (3, 4, 6, 3) bottleneck blocks of widths M = width, 2 width, 4 width, 8 width, each
    leaving with 4 M channels; the first block of a stage has a projection shortcut and, from the second stage on,
    stride 2 on its 3x3 convolution.  The input is the stem's output ([batch][width][H][W], 64 x 56 x 56 for the
    real network); the stem, pooling and classifier are dense layers outside this library.  Weights are seeded and
    synthetic (make_block_weights), ranks come from ``rank(M)``."""

    def __init__(self, batch: int, H: int = 56, W: int = 56, width: int = 64, blocks=(3, 4, 6, 3), rank=default_rank,
                 seed: int = 0, device: int = 0, layout: int = B.LAYOUT_NCHW, tunings=None):
        import torch
        self.dev = torch.device("cuda", device)
        self.layout = layout
        self.batch, self.width = batch, width
        self.blocks = []
        self.weights = []
        C, h, w = width, H, W
        for stage, count in enumerate(blocks):
            M = width << stage
            for i in range(count):
                first = i == 0
                stride = 2 if (first and stage > 0) else 1
                R = rank(M)
                wts = make_block_weights(C, M, R, R, seed + 100 * stage + i, C_out=4 * M, projection=first)
                blk = TuckerBottleneck(batch, C, M, h, w, R, R, wts, device, layout, stride=stride, C_out=4 * M, tunings=tunings)
                assert blk.projection == first
                self.blocks.append(blk)
                self.weights.append(wts)
                C, h, w = 4 * M, blk.l2.Ho, blk.l2.Wo
        self.in_shape = (batch, H, W, width) if layout == B.LAYOUT_NHWC else (batch, width, H, W)
        self.y = self.blocks[-1].y

    def __call__(self, x):
        """Enqueue every block on the current stream; returns the last block's (network-owned) output."""
        for blk in self.blocks:
            x = blk(x)
        return x

    def capture(self, x_static):
        """One HIP graph holding every launch of the network on x_static."""
        import torch
        self(x_static)                       # once eagerly: kernel attributes, lazy module load
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            x = x_static
            for blk in self.blocks:
                blk.bind(x)                  # launchers carry their stream: bind to the capturing one
                x = blk()
        for blk in self.blocks:
            blk._launchers = None
        return graph

    def kernels(self) -> int:
        return sum(b.kernels() for b in self.blocks)

    def flops(self) -> int:
        return sum(b.flops() for b in self.blocks)

    def describe(self) -> str:
        return "\n".join("block %2d  %s" % (i, b.describe()) for i, b in enumerate(self.blocks))

    def close(self) -> None:
        for b in self.blocks:
            b.close()


class TuckerResNet18Body(TuckerResNetBody):
    """The four residual stages of a ResNet-18-shaped network: ``blocks`` = (2, 2, 2, 2) basic blocks of widths width,
    2 width, 4 width, 8 width, every 3x3 convolution in Tucker-2 form with ranks ``rank(channels)`` on each side (default
    a quarter of the channels: the ranks of the batch-1 benchmark sweep); from the second stage on the first block of a
    stage has stride 2 and a projection shortcut.  Input: the stem's output, [batch][width][H][W] (64 x 56 x 56)."""

    def __init__(self, batch: int, H: int = 56, W: int = 56, width: int = 64, blocks=(2, 2, 2, 2), rank=lambda ch: max(1, ch // 4),
                 seed: int = 0, device: int = 0, layout: int = B.LAYOUT_NCHW, tunings=None):
        import torch
        self.dev = torch.device("cuda", device)
        self.layout = layout
        self.batch, self.width = batch, width
        self.blocks = []
        self.weights = []
        C, h, w = width, H, W
        for stage, count in enumerate(blocks):
            M = width << stage
            for i in range(count):
                stride = 2 if (i == 0 and stage > 0) else 1
                Ra, Rb = (rank(C), rank(M)), (rank(M), rank(M))
                wts = make_basic_weights(C, M, Ra, Rb, seed + 100 * stage + i, projection=stride != 1 or M != C)
                blk = TuckerBasicBlock(batch, C, M, h, w, Ra, Rb, wts, device, layout, stride=stride, tunings=tunings)
                self.blocks.append(blk)
                self.weights.append(wts)
                C, h, w = M, blk.la.Ho, blk.la.Wo
        self.in_shape = (batch, H, W, width) if layout == B.LAYOUT_NHWC else (batch, width, H, W)
        self.y = self.blocks[-1].y


def oracle_tunings(layout: int = B.LAYOUT_NCHW, device: int = 0, iters: int = 100, progress=None):
    """A ``tunings`` function for the blocks and networks above that replaces the selector's closed-form choice by
    exhaustive search, the paper's "oracle" setting next to its "modeling" one (section 7): the first time a convolution
    shape is asked for, every launchable tuning of it is timed on the GPU (Tucker layers: autotune.autotune, 500-2400
    tunings; dense layers: the 36 register-tile / wavefront combinations, with the epilogue the layer will run with),
    the fastest is kept and served from then on.  Returns (function, log) -- log lists (kind, layer, model us, best us)."""
    import torch
    from .autotune import _time, autotune
    cache, log = {}, []

    def dense(layer, epilogue):
        dev = torch.device("cuda", device)
        x = torch.randn((layer.batch, layer.H, layer.W, layer.C) if layout == B.LAYOUT_NHWC else (layer.batch, layer.C, layer.H, layer.W), device=dev)
        W = torch.randn((layer.C, layer.N, layer.K, layer.K), device=dev) * float(layer.C * layer.K * layer.K) ** -0.5
        rows = []
        for tun in [None] + [dict(mb=(0, mb, 0), pb=(0, pb, 0), waves=(0, nw, 0)) for mb in (1, 2, 4) for pb in (1, 2, 4) for nw in (1, 2, 4, 8)]:
            try:
                conv = DenseConv2d(layer, device, B.make_tuning(**tun) if tun else None, layout=layout)
            except B.TdcError:
                continue
            try:
                conv.pack(W)
                y = torch.empty(conv.out_shape(), device=dev)
                launch = conv.bind(x, y, bias=torch.zeros(layer.N, device=dev) if epilogue[0] else None,
                                   residual=torch.zeros_like(y) if epilogue[1] else None, relu=epilogue[2])
                rows.append((_time(launch, iters), tun is None, B.tdc_plan_get_tuning(conv.plan)))
                torch.cuda.synchronize()
            finally:
                conv.close()
        best = min(rows, key=lambda r: r[0])
        return [r for r in rows if r[1]][0][0], best[0], best[2]

    def pick(kind, layer, epilogue):
        key = (kind, layer.name(), epilogue if kind == "dense" else None)
        if key not in cache:
            if kind == "dense":
                model_us, best_us, tuning = dense(layer, epilogue)
            else:
                r = autotune(layer, device, iters=iters, layout=layout)
                model_us, best_us = r["auto"]["us"], r["best"]["us"]
                d = r["best"]["tuning"]
                tuning = B.make_tuning(variant={v: k for k, v in B.VARIANT_NAMES.items()}[d["variant"]], tile_h=d["tile_h"], tile_w=d["tile_w"],
                                       waves=tuple(d["waves"]), mb=tuple(d["mb"]), pb=tuple(d["pb"]))
            cache[key] = tuning
            log.append((kind, layer.name(), model_us, best_us))
            if progress:
                progress("%-6s %-44s model %6.2f us  best %6.2f us" % (kind, layer.name(), model_us, best_us))
        return cache[key]

    return pick, log


def time_network(net, iters: int = 100, repeats: int = 5) -> Dict[str, float]:
    """Median over ``repeats`` of the time per pass (HIP events around ``iters`` passes), eagerly and from one graph."""
    import torch
    x = torch.randn(net.in_shape, device=net.dev)
    graph = net.capture(x)

    def timed(fn):
        for _ in range(10):
            fn()
        out = []
        for _ in range(repeats):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                fn()
            b.record()
            b.synchronize()
            out.append(a.elapsed_time(b) * 1e3 / iters)
        return sorted(out)

    eager, replay = timed(lambda: net(x)), timed(graph.replay)
    torch.cuda.synchronize()
    del graph
    return {"eager_us": eager[len(eager) // 2], "eager_us_min": eager[0], "eager_us_max": eager[-1],
            "graph_us": replay[len(replay) // 2], "graph_us_min": replay[0], "graph_us_max": replay[-1]}


def main(argv=None) -> int:
    import torch
    if not torch.cuda.is_available():
        sys.exit("bottleneck needs a GPU")
    B.load()
    layout = B.LAYOUT_NHWC if argv and "--nhwc" in argv else B.LAYOUT_NCHW
    if argv and ("--resnet50" in argv or "--resnet18" in argv):
        batch = int(argv[argv.index("--batch") + 1]) if "--batch" in argv else 1
        deep = "--resnet50" in argv
        cls = TuckerResNetBody if deep else TuckerResNet18Body
        net = cls(batch, layout=layout)
        r = time_network(net)
        print(net.describe())
        print("ResNet-%d body, batch %d, %s: %d blocks, %d kernels, %.3f GFLOP; eager %.1f us, one graph %.1f us" % (
            50 if deep else 18, batch, "NHWC" if layout else "NCHW", len(net.blocks), net.kernels(), net.flops() / 1e9,
            r["eager_us"], r["graph_us"]), flush=True)
        net.close()
        if "--oracle" in argv:       # the same network with every convolution's tuning found by exhaustive search
            pick, log = oracle_tunings(layout, progress=lambda m: print("   " + m, flush=True))
            tuned = cls(batch, layout=layout, tunings=pick)
            ro = time_network(tuned)
            print(tuned.describe())
            print("... with exhaustively searched tunings (%d shapes searched): %d kernels; eager %.1f us, one graph %.1f us; "
                  "the selector's network is %.1f %% behind" % (len(log), tuned.kernels(), ro["eager_us"], ro["graph_us"],
                                                              100 * (r["eager_us"] / ro["eager_us"] - 1)), flush=True)
            tuned.close()
        return 0
    print("%-34s %8s %10s %10s  %s" % ("block (batch 1, %s)" % ("NHWC" if layout else "NCHW"), "kernels", "eager us", "graph us", "plans"),
          flush=True)
    for (C, M, HW, R) in ((256, 64, 56, 16), (512, 128, 28, 32), (1024, 256, 14, 64), (2048, 512, 7, 128)):
        blk = TuckerBottleneck(1, C, M, HW, HW, R, R, make_block_weights(C, M, R, R, 7), layout=layout)
        x = torch.randn((1, HW, HW, C) if layout else (1, C, HW, HW), device=blk.dev)
        graph = blk.capture(x)

        def timed(fn, iters=300):
            for _ in range(20):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                fn()
            b.record()
            b.synchronize()
            return a.elapsed_time(b) * 1e3 / iters

        eager, replay = timed(blk), timed(graph.replay)
        print("%-34s %8d %10.2f %10.2f  %s" % ("C=%d M=%d %dx%d r=%d" % (C, M, HW, HW, R), blk.kernels(), eager, replay,
                                             blk.describe()), flush=True)
        torch.cuda.synchronize()
        blk.close()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
