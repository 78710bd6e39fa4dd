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

    python -m paper_2211_03715_amd.bottleneck [--nhwc]   # eager vs graph latency of a few block shapes
"""
from __future__ import annotations

import sys
from typing import Dict

import numpy as np

from . import binding as B
from .layer import DenseConv2d, TuckerConv2d
from .workloads import Layer


def make_block_weights(C: int, M: int, R1: int, R2: int, seed: int) -> Dict[str, np.ndarray]:
    """Seeded float32 weights of one block, N(0, 1/fan_in); biases N(0, 0.01)."""
    rng = np.random.default_rng(seed)
    n = lambda shape, fan: (rng.standard_normal(shape, dtype=np.float32) * np.float32(fan ** -0.5))
    return {"W1": n((C, M, 1, 1), C), "b1": n((M,), 100.0),
            "U_in": n((M, R1), M), "core": n((R1, R2, 3, 3), R1 * 9), "U_out": n((R2, M), R2), "b2": n((M,), 100.0),
            "W3": n((M, C, 1, 1), M), "b3": n((C,), 100.0)}


class TuckerBottleneck:
    def __init__(self, batch: int, C: int, M: int, H: int, W: int, R1: int, R2: int, weights: Dict, device: int = 0,
                 layout: int = B.LAYOUT_NCHW):
        """``layout``: LAYOUT_NCHW (x, y [batch][C][H][W]) or LAYOUT_NHWC ([batch][H][W][C]); C, M multiples of 4 for NHWC."""
        import torch
        self.dev = torch.device("cuda", device)
        self.layout = layout
        self.l1 = Layer(batch, C, M, H, W, 1, 1, 1, 1, 0)
        self.l2 = Layer(batch, M, M, H, W, R1, R2, 3, 1, 1)
        self.l3 = Layer(batch, M, C, H, W, 1, 1, 1, 1, 0)
        self.w = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.dev) for k, v in weights.items()}
        self.conv1, self.conv2, self.conv3 = (DenseConv2d(self.l1, device, layout=layout), TuckerConv2d(self.l2, device, layout=layout),
                                              DenseConv2d(self.l3, device, layout=layout))
        self.conv1.pack(self.w["W1"])
        self.conv2.pack(self.w["U_in"], self.w["core"], self.w["U_out"])
        self.conv3.pack(self.w["W3"])
        self.t1 = torch.empty(self.conv1.out_shape(), device=self.dev, dtype=torch.float32)
        self.t2 = torch.empty(self.conv2.out_shape(), device=self.dev, dtype=torch.float32)
        self.y = torch.empty(self.conv3.out_shape(), device=self.dev, dtype=torch.float32)
        self._launchers = None
        self._x = None

    def bind(self, x):
        """Marshal the three calls for a fixed input tensor; returns self for chaining."""
        self._x = x
        self._launchers = (
            self.conv1.bind(x, self.t1, bias=self.w["b1"], relu=True),
            self.conv2.bind(self.t1, self.t2, bias=self.w["b2"], relu=True),
            self.conv3.bind(self.t2, self.y, bias=self.w["b3"], residual=x, relu=True),
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
        return 2 + self.conv2.kernel_count()

    def describe(self) -> str:
        return "1x1: %s | 3x3: %s | 1x1: %s" % (self.conv1.describe(), self.conv2.describe(), self.conv3.describe())

    def close(self) -> None:
        for c in (self.conv1, self.conv2, self.conv3):
            c.close()


def main(argv=None) -> int:
    import torch
    if not torch.cuda.is_available():
        sys.exit("bottleneck needs a GPU")
    B.load()
    layout = B.LAYOUT_NHWC if argv and "--nhwc" in argv else B.LAYOUT_NCHW
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
