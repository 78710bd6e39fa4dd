"""Phase timestamps of the one-launch kernels, read back from the probe build of the library.

    python -m paper_2211_03715_amd.build --probes                      # once: libtdc_probe.so
    python -m paper_2211_03715_amd.probes 32,128,256,56,56,32,64,3,2,1 [--nhwc] [--variant chain]

The kernels mark phase boundaries with TDC_PROBE(slot) (tdc_mfma.h).  One-launch kernels: 0 = kernel entry, 3 = end
of stage 1, 4 = after the barrier behind it, 5 = end of stage 2, 7 = end of the kernel.  GEMM kernels (split, merged,
dense): slots 5*(stage - 1) + {0: entry, 1: operands placed, 2: first loads issued, 3: MFMA loop done, 4: stored}.
merged_xcd: 0 entry, 1 stage-1 loads issued, 2 its MFMAs done, 3 z1 stored, 4 past the barrier, 5 loads of the merged
GEMM issued, 6 its MFMAs done, 7 end.
This prints, per pair of consecutive marks (in time order), the median / min / max time over all wavefronts of one
call and the shader clock in between -- which is how the per-phase budgets quoted in the design notes were taken.
"""
from __future__ import annotations

import argparse
import ctypes
import sys

import numpy as np

from . import binding as B
from .build import PROBE_LIB
from .workloads import Layer, make_inputs

def phase_times(layer: Layer, tuning=None, layout: int = B.LAYOUT_NCHW, iters: int = 50):
    """Runs the layer on the probe library.  Returns (plan description, event-timed us per launch,
    [(slot_a, slot_b, median, min, max)] in us for consecutive marks that were reached, shader GHz between them)."""
    import torch
    lib = B.load(PROBE_LIB)
    B._lib = lib                       # the convenience layer below goes through the probe library
    lib.tdc_debug_read_probes.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    from .layer import TuckerConv2d
    dev = torch.device("cuda:0")
    t = {k: torch.from_numpy(v).to(dev) for k, v in make_inputs(layer, 1).items()}
    conv = TuckerConv2d(layer, 0, tuning, layout=layout)
    try:
        if layout == B.LAYOUT_NHWC:
            t["x"] = t["x"].permute(0, 2, 3, 1).contiguous()
        y = torch.empty(conv.out_shape(), device=dev)
        conv.pack(t["U_in"], t["core"], t["U_out"])
        launch = conv.bind(t["x"], y)
        for _ in range(20):
            launch()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            launch()
        b.record()
        b.synchronize()
        if lib.tdc_debug_clear_probes() != 0:
            raise RuntimeError("could not clear the probe buffer")
        launch()                        # the marks of exactly one call
        torch.cuda.synchronize()
        n = 2 * 8 * 16 * 4096
        buf = np.zeros(n, dtype=np.uint64)
        if lib.tdc_debug_read_probes(buf.ctypes.data, n) != 0:
            raise RuntimeError("could not read the probe buffer")
        marks = buf.reshape(4096, 8, 16, 2).astype(np.int64)
        clk, wall = marks[..., 0], marks[..., 1]
        reached = [s for s in range(16) if (wall[:, :, s] > 0).any()]
        reached.sort(key=lambda s: np.median(wall[:, :, s][wall[:, :, s] > 0]))
        phases = []
        for s0, s1 in zip(reached[:-1], reached[1:]):
            both = (wall[:, :, s0] > 0) & (wall[:, :, s1] > 0)
            if not both.any():
                continue
            dt = (wall[:, :, s1] - wall[:, :, s0])[both] / 100.0
            ghz = float(np.median((clk[:, :, s1] - clk[:, :, s0])[both] / np.maximum((wall[:, :, s1] - wall[:, :, s0])[both], 1))) / 10.0
            phases.append((s0, s1, float(np.median(dt)), float(dt.min()), float(dt.max()), ghz))
        return conv.describe(), a.elapsed_time(b) * 1e3 / iters, phases
    finally:
        conv.close()


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("shapes", nargs="+", metavar="B,C,N,H,W,R1,R2[,K,stride,pad]")
    ap.add_argument("--nhwc", action="store_true")
    ap.add_argument("--variant", default="auto", choices=["auto", "fused", "chain", "fused_merged", "merged", "merged_xcd", "split"])
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        sys.exit("probes needs a GPU")
    variant = {"auto": None, "fused": B.VARIANT_FUSED, "chain": B.VARIANT_CHAIN, "fused_merged": B.VARIANT_FUSED_MERGED,
               "merged": B.VARIANT_MERGED, "merged_xcd": B.VARIANT_MERGED_XCD, "split": B.VARIANT_SPLIT}[args.variant]
    for spec in args.shapes:
        L = Layer(*[int(v) for v in spec.split(",")])
        desc, us, phases = phase_times(L, B.make_tuning(variant=variant) if variant else None,
                                       B.LAYOUT_NHWC if args.nhwc else B.LAYOUT_NCHW)
        print("%s %s: %s\n   %.2f us per call (probe build)" % (L.name(), "nhwc" if args.nhwc else "nchw", desc, us), flush=True)
        for s0, s1, med, lo, hi, ghz in phases:
            print("   mark %2d -> %2d   median %6.2f us   min %6.2f   max %6.2f   shader clock %.2f GHz" % (s0, s1, med, lo, hi, ghz), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
