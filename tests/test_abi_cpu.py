"""The C-ABI library without a GPU: it loads, exports what the header declares, and its host
logic (validation, status strings, output-size rule, selector) behaves.  No compute calls."""
import ctypes
import os
import re

import pytest

from paper_2211_03715_amd import binding as B
from paper_2211_03715_amd.workloads import config_layers

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tdc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    lib = B.load()
    names = _declared()
    assert "tdc_conv_tucker2" in names and "tdc_plan_create" in names and "tdc_plan_destroy" in names
    for n in names:
        assert hasattr(lib, n), "libtdc.so does not export %s" % n
    assert sorted(B.EXPORTS) == names, "binding.EXPORTS and include/*.h disagree"
    for n in names:
        assert hasattr(B, n), "binding has no wrapper named %s" % n


def test_struct_layouts_match_header():
    assert ctypes.sizeof(B.tdc_shape) == 11 * 4
    assert ctypes.sizeof(B.tdc_tuning) == 12 * 4


def test_status_strings_and_version():
    assert B.tdc_version() >= 100
    seen = set()
    for code in range(0, -8, -1):
        s = B.status_string(code)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert B.status_string(-99) == "unknown status"


def test_out_size_rule():
    assert B.tdc_out_size(56, 3, 1, 1) == 56
    assert B.tdc_out_size(56, 3, 2, 1) == 28
    assert B.tdc_out_size(7, 3, 2, 1) == 4
    assert B.tdc_out_size(5, 3, 1, 0) == 3
    assert B.tdc_out_size(2, 3, 1, 0) == 0
    assert B.tdc_out_size(0, 3, 1, 1) == 0


def _create(shape, tuning=None):
    lib = B.load()
    plan = ctypes.c_void_p()
    if tuning is None:
        rc = lib.tdc_plan_create(ctypes.byref(plan), ctypes.byref(shape), 0)
    else:
        rc = lib.tdc_plan_create_tuned(ctypes.byref(plan), ctypes.byref(shape), 0, ctypes.byref(tuning))
    return rc, plan


def test_validation_happens_before_any_device_call():
    lib = B.load()
    assert lib.tdc_plan_create(None, None, 0) == B.TDC_ERR_NULL
    bad = [B.make_shape(0, 4, 4, 8, 8, 2, 2), B.make_shape(1, 0, 4, 8, 8, 2, 2), B.make_shape(1, 4, 4, 8, 8, 0, 2),
           B.make_shape(1, 4, 4, 8, 8, 2, 2, K=3, stride=0), B.make_shape(1, 4, 4, 8, 8, 2, 2, K=3, pad=-1),
           B.make_shape(1, 4, 4, 2, 8, 2, 2, K=3, pad=0), B.make_shape(1, 4, 4, 8, 8, 2, 2, K=0)]
    for s in bad:
        rc, plan = _create(s)
        assert rc == B.TDC_ERR_BAD_SHAPE and not plan.value
    unsupported = [B.make_shape(1, 4, 4, 8, 8, 2, 2, layout=2), B.make_shape(1, 4, 4, 8, 8, 2, 2, layout=-1),
                   B.make_shape(1, 6, 4, 8, 8, 2, 2, layout=B.LAYOUT_NHWC), B.make_shape(1, 4, 6, 8, 8, 2, 2, layout=B.LAYOUT_NHWC),
                   B.make_shape(1, 4, 4, 8, 8, 2, 2, K=9, pad=4),
                   B.make_shape(1, 4, 4, 8, 8, 2, 2, stride=5), B.make_shape(1, 4, 4, 8, 8, 2, 2, K=3, pad=3),
                   B.make_shape(4096, 1024, 4, 1024, 1024, 2, 2),
                   B.make_shape(1, 8, 600, 1024, 1024, 2, 2),       # one output image of 2.3 GiB: more than a buffer descriptor spans
                   B.make_shape(1, 600, 8, 1024, 1024, 2, 2)]       # the same for one input image
    for s in unsupported:
        rc, plan = _create(s)
        assert rc == B.TDC_ERR_UNSUPPORTED and not plan.value
    # calls on a NULL plan
    s = B.make_shape(1, 4, 4, 8, 8, 2, 2)
    assert lib.tdc_conv_tucker2(None, None, None, None, None, None, None, ctypes.byref(s)) == B.TDC_ERR_NULL
    assert lib.tdc_plan_pack_weights(None, None, None, None, None) == B.TDC_ERR_NULL
    assert lib.tdc_plan_destroy(None) == B.TDC_OK
    assert lib.tdc_plan_get_tuning(None, None) == B.TDC_ERR_NULL
    assert lib.tdc_plan_workspace_bytes(None) == 0


def test_selector_fills_a_launchable_tuning_for_every_workload():
    for cfg in range(1, 8):
        for L in config_layers(cfg):
            t = B.tdc_select_tuning(B.make_shape(**L.asdict()))
            n = B.tdc_select_tuning(B.make_shape(**L.asdict(), layout=B.LAYOUT_NHWC)).as_dict()
            assert n["variant"] in ("split", "fused", "chain", "merged", "fused_merged"), n
            if L.batch == 1 and cfg <= 6:
                assert n == t.as_dict()        # on these layers the latency-regime estimates pick the same plan in both layouts
            d = t.as_dict()
            assert d["variant"] in ("split", "fused", "chain", "merged", "fused_merged"), d
            assert all(1 <= w <= 8 for w in d["waves"]) and all(1 <= m <= 8 for m in d["mb"])
            if d["variant"] in ("fused", "chain", "fused_merged"):
                assert 1 <= d["tile_h"] <= L.Ho and 1 <= d["tile_w"] <= L.Wo


def test_selector_respects_forced_fields_and_rejects_misfits():
    L = config_layers(1)[0]
    s = B.make_shape(**L.asdict())
    t = B.tdc_select_tuning(s, tuning=B.make_tuning(variant=B.VARIANT_FUSED, tile_h=8, tile_w=8, waves=(4, 0, 0)))
    assert (t.variant, t.tile_h, t.tile_w, t.waves[0]) == (B.VARIANT_FUSED, 8, 8, 4)
    t = B.tdc_select_tuning(s, tuning=B.make_tuning(variant=B.VARIANT_SPLIT, mb=(1, 1, 4), pb=(2, 2, 1)))
    assert t.variant == B.VARIANT_SPLIT and list(t.mb) == [1, 1, 4] and list(t.pb) == [2, 2, 1]
    with pytest.raises(B.TdcError):   # register tiles must divide the 16-channel blocks (R1 = 16 is one block)
        B.tdc_select_tuning(s, tuning=B.make_tuning(variant=B.VARIANT_SPLIT, mb=(2, 1, 4)))
    with pytest.raises(B.TdcError) as e:
        B.tdc_select_tuning(s, tuning=B.make_tuning(variant=B.VARIANT_SPLIT, mb=(3, 1, 1)))
    assert e.value.status == B.TDC_ERR_BAD_TUNING
    with pytest.raises(B.TdcError):   # LDS budget too small for any fused tile
        B.tdc_select_tuning(s, lds_bytes=2048, tuning=B.make_tuning(variant=B.VARIANT_FUSED))
    with pytest.raises(B.TdcError):
        B.tdc_select_tuning(s, tuning=B.make_tuning(variant=9))


def test_selector_throughput_regime_counts_residency_by_registers():
    """Where the pixels alone fill the chip the choice is between FUSED and CHAIN, and the estimate counts the
    workgroups a compute unit holds by the kernels' register footprint (8 wavefronts of the chain kernel, not
    32): on a layer with two large tiles per compute unit, one 8-wavefront workgroup run twice and two
    4-wavefront ones run together get the same estimate, and the tie goes to the pair -- the tuning the sweeps
    found faster."""
    for layout in (B.LAYOUT_NCHW, B.LAYOUT_NHWC):
        s = B.make_shape(64, 64, 64, 56, 56, 16, 16, layout=layout)
        d = B.tdc_select_tuning(s, tuning=B.make_tuning(variant=B.VARIANT_CHAIN)).as_dict()
        tiles = -(-56 // d["tile_h"]) * -(-56 // d["tile_w"]) * 64
        assert tiles > 256 and d["waves"][0] == 4, d            # more tiles than compute units: pairs of 4 wavefronts
        assert B.tdc_select_tuning(s).as_dict()["variant"] in ("fused", "chain")
    # one tile per compute unit: the whole CU goes to one 8-wavefront workgroup
    d = B.tdc_select_tuning(B.make_shape(32, 128, 128, 28, 28, 32, 32), tuning=B.make_tuning(variant=B.VARIANT_CHAIN)).as_dict()
    assert -(-28 // d["tile_h"]) * -(-28 // d["tile_w"]) * 32 <= 256 and d["waves"][0] == 8, d
    # NCHW rows that are read in 16-byte runs get tiles whose width is a multiple of 4
    d = B.tdc_select_tuning(B.make_shape(32, 128, 256, 56, 56, 32, 64, 3, 2, 1)).as_dict()
    assert d["variant"] == "chain" and d["tile_w"] % 4 == 0, d
    # below the threshold (batch x output pixels < 16 per compute unit) neither the chain kernel nor that rule applies
    assert B.tdc_select_tuning(B.make_shape(1, 128, 128, 28, 28, 32, 32)).as_dict()["variant"] != "chain"


def test_selector_handles_the_dense_layer():
    lib = B.load()
    for cfg in (2, 4):
        for L in config_layers(cfg):
            t = B.tdc_select_tuning(B.make_shape(**L.asdict()), tuning=B.make_tuning(variant=B.VARIANT_DENSE))
            d = t.as_dict()
            assert d["variant"] == "dense" and d["mb"][1] in (1, 2, 4) and 1 <= d["waves"][1] <= 8, d
            assert ((L.N + 15) // 16) % d["mb"][1] == 0
    s = B.make_shape(1, 40, 24, 9, 9, 1, 1)           # N = 24 is two 16-blocks: a tile of four cannot divide it
    with pytest.raises(B.TdcError):
        B.tdc_select_tuning(s, tuning=B.make_tuning(variant=B.VARIANT_DENSE, mb=(0, 4, 0)))
    assert lib.tdc_conv_dense(None, None, None, None, None, ctypes.byref(s)) == B.TDC_ERR_NULL
    assert lib.tdc_plan_pack_dense(None, None, None) == B.TDC_ERR_NULL


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(RuntimeError):
        B.load(str(tmp_path / "libtdc.so"))


def test_constant_division_matches_integer_division(tmp_path):
    """The kernels divide by launch-time constants with a precomputed multiplier (csrc/tdc_div.h).
    A host program built from that header compares it with `/` for every divisor up to 4096 (and a
    few large ones) on all dividends below 2^16, a dense band around every multiple of the divisor
    near 2^31, and 2^20 pseudo-random 32-bit dividends."""
    import shutil
    import subprocess
    cxx = shutil.which("g++")
    assert cxx, "g++ is needed for this test"
    src = tmp_path / "divcheck.cpp"
    src.write_text(r'''
#include <cstdio>
#include <cstdint>
#include "tdc_div.h"
static int check(unsigned d, unsigned x, const TdcDiv &c) {
    const unsigned t = (unsigned)(((uint64_t)c.m * x) >> 32);
    if (tdc_div_from_hi(x, t, c) != x / d) { std::printf("d=%u x=%u\n", d, x); return 1; }
    return 0;
}
int main() {
    unsigned big[] = {4097u, 12345u, 65535u, 65536u, 65537u, 1000003u, 0x3fffffffu, 0x40000000u, 0x7fffffffu};
    uint64_t bad = 0, n = 0;
    for (unsigned i = 1; i <= 4096 + sizeof big / sizeof *big; ++i) {
        const unsigned d = i <= 4096 ? i : big[i - 4097];
        const TdcDiv c = tdc_make_div(d);
        for (unsigned x = 0; x < 65536; ++x, ++n) bad += check(d, x, c);
        const unsigned q = 0x80000000u / d;
        for (unsigned k = (q > 2 ? q - 2 : 0); k <= q + 2; ++k)
            for (int o = -2; o <= 2; ++o, ++n) bad += check(d, (unsigned)((uint64_t)k * d + o), c);
        bad += check(d, 0xffffffffu, c) + check(d, 0x7fffffffu, c);
        uint64_t s = 0x9e3779b97f4a7c15ull * d;
        for (int r = 0; r < 256; ++r, ++n) { s = s * 6364136223846793005ull + 1442695040888963407ull; bad += check(d, (unsigned)(s >> 32), c); }
    }
    std::printf("checked %llu bad %llu\n", (unsigned long long)n, (unsigned long long)bad);
    return bad != 0;
}
''')
    exe = tmp_path / "divcheck"
    inc = os.path.join(os.path.dirname(B.__file__), "csrc")
    subprocess.run([cxx, "-O2", "-I", inc, str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout[-2000:]


def test_paper_tile_rule_orders_by_computation_then_by_data_movement():
    """Host logic of the offline analysis: the paper's rule keeps the tilings of least computation latency
    (waves x per-block latency, halo included) and among those takes the one that moves the fewest bytes."""
    from paper_2211_03715_amd.autotune import paper_tile_rule
    from paper_2211_03715_amd.workloads import Layer
    L = Layer(1, 64, 64, 56, 56, 16, 16)

    def row(th, tw, nw, lds, us):
        return {"us": us, "plan": "fused tile=%dx%d lds=%dB" % (th, tw, lds),
                "tuning": {"variant": "fused", "tile_h": th, "tile_w": tw, "waves": [nw] * 3, "mb": [1, 1, 1], "pb": [1, 1, 1]}}

    # one resident workgroup per CU (100 KB of LDS).  7x8 and 8x7 tiles: 56 workgroups, one wave of blocks,
    # the same halo area -> the same computation latency and the same traffic.  14x8: 28 workgroups, also one
    # wave, but each block has about twice the FLOPs -> more computation latency, fewer bytes moved.
    rows = [row(7, 8, 4, 100000, 3.0), row(8, 7, 4, 100000, 2.0), row(14, 8, 4, 100000, 1.0)]
    assert paper_tile_rule(L, rows, top=0.05)["tuning"]["tile_h"] in (7, 8)       # step 1 decides, whatever the timings
    pick = paper_tile_rule(L, rows, top=1.0)                                      # all kept: step 2 decides
    assert (pick["tuning"]["tile_h"], pick["tuning"]["tile_w"]) == (14, 8)
    # two waves of blocks double the latency: 1x8 tiles (392 workgroups) lose to 2x8 tiles (196) of twice the block size
    # only if a block's latency less than doubles -- it does (halo rows 3 -> 4), so step 1 prefers 2x8
    rows = [row(1, 8, 4, 100000, 1.0), row(2, 8, 4, 100000, 2.0)]
    assert paper_tile_rule(L, rows, top=0.05)["tuning"]["tile_h"] == 2
    assert paper_tile_rule(L, [r for r in rows if r["tuning"]["variant"] != "fused"]) == {}
