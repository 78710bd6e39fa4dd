"""GPU parity of the fused output epilogue (bias, residual, ReLU) of tdc_conv_tucker2_ex and
tdc_conv_dense_ex against the oracle, for every kernel family."""
import sys

import numpy as np
import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.workloads import Layer, make_dense_inputs, make_inputs
from parity_util import assert_parity

pytestmark = pytest.mark.gpu

VARIANTS = {"naive": B.VARIANT_NAIVE, "split": B.VARIANT_SPLIT, "fused": B.VARIANT_FUSED, "chain": B.VARIANT_CHAIN,
            "merged": B.VARIANT_MERGED, "fused_merged": B.VARIANT_FUSED_MERGED, "auto": B.VARIANT_AUTO}
LAYERS = [Layer(2, 20, 24, 19, 23, 17, 33), Layer(1, 64, 64, 56, 56, 16, 16), Layer(3, 33, 18, 12, 40, 8, 40, 3, 2, 1),
          Layer(2, 32, 40, 8, 12, 16, 16)]     # the last one: tile and image widths multiples of 4 (16-byte stores in CHAIN)
EPILOGUES = [dict(bias=True, residual=False, relu=False), dict(bias=False, residual=False, relu=True),
             dict(bias=False, residual=True, relu=False), dict(bias=True, residual=True, relu=True)]


def _announce(*parts):
    print("[case]", *parts, flush=True)
    sys.stdout.flush()


def _epilogue_inputs(layer, seed):
    rng = np.random.default_rng(seed)
    Ho, Wo = layer.Ho, layer.Wo
    return (rng.standard_normal(layer.N, dtype=np.float32),
            rng.standard_normal((layer.batch, layer.N, Ho, Wo), dtype=np.float32))


@pytest.mark.parametrize("epi", EPILOGUES, ids=lambda e: "+".join(k for k, v in e.items() if v))
@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: l.name())
def test_tucker_epilogue(orc, layer, variant, epi):
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    _announce("epilogue", variant, layer.name(), epi)
    inputs = make_inputs(layer, 321)
    bias, res = _epilogue_inputs(layer, 654)
    want, _ = orc.conv_factored(orc.Shape(**layer.asdict()), **inputs)
    want = orc.apply_epilogue(want, bias if epi["bias"] else None, res if epi["residual"] else None, epi["relu"])
    dev = torch.device("cuda:0")
    t = {k: torch.from_numpy(v).to(dev) for k, v in inputs.items()}
    tb, tr = torch.from_numpy(bias).to(dev), torch.from_numpy(res).to(dev)
    conv = TuckerConv2d(layer, 0, B.make_tuning(variant=VARIANTS[variant]))
    try:
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.full((layer.batch, layer.N, conv.Ho, conv.Wo), float("nan"), device=dev)
        conv(t["x"], y, bias=tb if epi["bias"] else None, residual=tr if epi["residual"] else None, relu=epi["relu"])
        torch.cuda.synchronize()
        assert_parity(y.cpu().numpy(), want, "%s %s [%s]" % (variant, layer.name(), conv.describe()))
        # the bound launcher takes the same epilogue
        y2 = torch.full_like(y, float("nan"))
        conv.bind(t["x"], y2, bias=tb if epi["bias"] else None, residual=tr if epi["residual"] else None, relu=epi["relu"])()
        torch.cuda.synchronize()
        assert torch.equal(y, y2)
    finally:
        conv.close()


@pytest.mark.parametrize("epi", EPILOGUES, ids=lambda e: "+".join(k for k, v in e.items() if v))
@pytest.mark.parametrize("layer", [Layer(2, 20, 24, 19, 23, 1, 1), Layer(1, 64, 256, 14, 14, 1, 1, 1, 1, 0)],
                         ids=lambda l: l.name())
def test_dense_epilogue(orc, layer, epi):
    import torch
    from paper_2211_03715_amd.layer import DenseConv2d
    _announce("dense epilogue", layer.name(), epi)
    inputs = make_dense_inputs(layer, 987)
    bias, res = _epilogue_inputs(layer, 654)
    want, _ = orc.conv_dense_with(orc.Shape(**layer.asdict()), inputs["x"], inputs["W"].astype(np.float64))
    want = orc.apply_epilogue(want, bias if epi["bias"] else None, res if epi["residual"] else None, epi["relu"])
    dev = torch.device("cuda:0")
    x, W = torch.from_numpy(inputs["x"]).to(dev), torch.from_numpy(inputs["W"]).to(dev)
    tb, tr = torch.from_numpy(bias).to(dev), torch.from_numpy(res).to(dev)
    conv = DenseConv2d(layer, 0)
    try:
        conv.pack(W)
        y = torch.full((layer.batch, layer.N, conv.Ho, conv.Wo), float("nan"), device=dev)
        conv(x, y, bias=tb if epi["bias"] else None, residual=tr if epi["residual"] else None, relu=epi["relu"])
        torch.cuda.synchronize()
        assert_parity(y.cpu().numpy(), want, "dense %s [%s]" % (layer.name(), conv.describe()))
    finally:
        conv.close()
