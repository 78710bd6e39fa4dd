"""Are the pins sharp?  Plant one plausible mistake at a time in a copy of the oracle's C source
(a dropped term, a flipped kernel, a transposed operand, a wrong bound), build it on the CPU and
require that at least one pin fails.  Nothing here touches a GPU."""
import os
import subprocess

import pytest

from oracle_pins import ALL_PINS

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "tdc_oracle.c")

# (name, function the edit is made in or None for every occurrence, text to find, replacement)
MUTANTS = [
    ("core_flipped_kernel", "orc_core", "i * st + r - pad", "i * st + (K - 1 - r) - pad"),
    ("flip_in_core_and_dense", None, "j * st + s - pad", "j * st + (K - 1 - s) - pad"),
    ("core_rs_swapped", "orc_core", "* K + r) * K + s]", "* K + s) * K + r]"),
    ("core_modes_transposed", "orc_core", "((size_t)d1 * R2 + d2)", "((size_t)d2 * R1 + d1)"),
    ("core_modes_transposed_everywhere", None, "((size_t)d1 * R2 + d2)", "((size_t)d2 * R1 + d1)"),
    ("core_pad_ignored", "orc_core", "i * st + r - pad", "i * st + r"),
    ("pad_ignored_everywhere", None, "+ r - pad", "+ r"),
    ("core_stride_dropped", "orc_core", "i * st + r - pad", "i + r - pad"),
    ("stride_dropped_everywhere", None, "j * st + s", "j + s"),
    ("core_dropped_rank_term", "orc_core", "d1 < R1", "d1 < R1 - 1"),
    ("core_dropped_tap", "orc_core", "s < K", "s < K - 1"),
    ("stage1_uin_transposed", "orc_stage1", "U_in[(size_t)c * R1 + d1]", "U_in[(size_t)d1 * C + c]"),
    ("uin_transposed_everywhere", None, "U_in[(size_t)c * R1 + d1]", "U_in[(size_t)d1 * sh->C + c]"),
    ("stage1_dropped_channel", "orc_stage1", "c < C", "c < C - 1"),
    ("stage3_uout_transposed", "orc_stage3", "U_out[(size_t)d2 * N + n]", "U_out[(size_t)n * R2 + d2]"),
    ("uout_transposed_everywhere", None, "U_out[(size_t)d2 * N + n]", "U_out[(size_t)n * sh->R2 + d2]"),
    ("stage3_dropped_term", "orc_stage3", "d2 < R2", "d2 < R2 - 1"),
    ("stage3_sign", "orc_stage3", "acc += zv", "acc -= zv"),
    ("dense_wd_transposed", "orc_conv_dense", "((size_t)c * N + n)", "((size_t)n * C + c)"),
    ("dense_dropped_channel", "orc_conv_dense", "c < C", "c < C - 1"),
    ("reconstruct_rs_swapped", "orc_reconstruct", "* K + r) * K + s];", "* K + s) * K + r];"),
    ("reconstruct_dropped_term", "orc_reconstruct", "d2 < R2", "d2 < R2 - 1"),
    ("out_size_off_by_one", None, "/ s->stride + 1", "/ s->stride"),
    ("out_size_ignores_pad", None, "s->H + 2 * s->pad - s->K) / s->stride",
     "s->H + s->pad - s->K) / s->stride"),
    ("batch_offset_dropped_in_core", "orc_core", "z1[(((size_t)b * R1 + d1)", "z1[(((size_t)0 * R1 + d1)"),
    ("padding_wraps_rows", "orc_core", "if (h < 0 || h >= H || w < 0 || w >= W) continue;",
     "if (h < 0 || h >= H) continue; if (w < 0) w += W; if (w >= W) w -= W;"),
]


def _mutate(text, func, old, new):
    if func is None:
        assert old in text, old
        return text.replace(old, new)
    start = text.index(" %s(" % func)
    end = text.index("\n}\n", start)
    body = text[start:end]
    assert old in body, (func, old)
    return text[:start] + body.replace(old, new) + text[end:]


@pytest.mark.parametrize("name,func,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(orc, tmp_path, name, func, old, new):
    text = _mutate(open(SRC).read(), func, old, new).replace("const int w =", "int w =")
    src = tmp_path / (name + ".c")
    src.write_text(text)
    out = tmp_path / ("lib%s.so" % name)
    subprocess.run(["gcc", "-std=c99", "-O1", "-fopenmp", "-fPIC", "-shared", "-o", str(out), str(src)],
                   check=True)
    lib = orc.load(str(out))
    caught = []
    for pin in ALL_PINS:
        try:
            pin(orc, lib)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin notices the planted mistake %r" % name
