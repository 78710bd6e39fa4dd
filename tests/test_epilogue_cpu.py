"""The oracle's output epilogue against hand-worked values, and the ABI's epilogue struct."""
import ctypes

import numpy as np

from oracle import tdc_oracle as orc
from paper_2211_03715_amd import binding as B


def test_oracle_epilogue_handworked():
    y = np.array([[[[1.0, -2.0]], [[-3.0, 4.0]]]])          # batch 1, N = 2, 1 x 2 pixels
    r = np.array([[[[1.0, 1.0]], [[1.0, -5.0]]]])
    assert orc.apply_epilogue(y).tolist() == y.tolist()
    assert orc.apply_epilogue(y, bias=[10.0, -10.0]).ravel().tolist() == [11.0, 8.0, -13.0, -6.0]     # bias per channel
    assert orc.apply_epilogue(y, relu=True).ravel().tolist() == [1.0, 0.0, 0.0, 4.0]
    assert orc.apply_epilogue(y, residual=r).ravel().tolist() == [2.0, -1.0, -2.0, -1.0]
    # relu comes last: (4 - 10 - 5) -> 0, (1 + 10 + 1) -> 12
    assert orc.apply_epilogue(y, bias=[10.0, -10.0], residual=r, relu=True).ravel().tolist() == [12.0, 9.0, 0.0, 0.0]
    assert y.ravel().tolist() == [1.0, -2.0, -3.0, 4.0]     # input untouched


def test_epilogue_struct_layout_and_null_handling():
    assert ctypes.sizeof(B.tdc_epilogue) == 24
    lib = B.load()
    s = B.make_shape(1, 4, 4, 8, 8, 2, 2)
    assert lib.tdc_conv_tucker2_ex(None, None, None, None, None, None, None, ctypes.byref(s), None) == B.TDC_ERR_NULL
    assert lib.tdc_conv_dense_ex(None, None, None, None, None, ctypes.byref(s), None) == B.TDC_ERR_NULL
