"""ctypes front end of the CPU oracle (``tdc_oracle.c``)  --  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module.  It imports nothing from the GPU package and the GPU
package imports nothing from here.

The C file is compiled with gcc into ``libtdc_oracle.so`` next to it (``build()``);
``load()`` builds it on demand when the library is missing or older than the source.

Array conventions (paper section 3; NCHW storage):
  x      float32 [B][C][H][W]
  U_in   float32 [C][R1]          U1(c,d1) of Eq. 1 / Eq. 2
  core   float32 [R1][R2][K][K]   core(d1,d2,r,s) of Eq. 1 / Eq. 3
  U_out  float32 [R2][N]          U2(d2,n) of Eq. 4
  y      float64 [B][N][Ho][Wo]
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tdc_oracle.c")
_LIB = os.path.join(_HERE, "libtdc_oracle.so")


class OrcShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("batch", "C", "N", "H", "W", "R1", "R2", "K", "stride", "pad")]


@dataclass(frozen=True)
class Shape:
    """One Tucker-2 convolution layer.  Ranks R1, R2 are the paper's D1, D2."""
    batch: int
    C: int
    N: int
    H: int
    W: int
    R1: int
    R2: int
    K: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.K) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.K) // self.stride + 1

    def c_struct(self) -> OrcShape:
        return OrcShape(self.batch, self.C, self.N, self.H, self.W,
                        self.R1, self.R2, self.K, self.stride, self.pad)


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if (not force and os.path.exists(out)
            and os.path.getmtime(out) >= os.path.getmtime(src)):
        return out
    tmp = out + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", tmp, src]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


_lib = None


def load(path: str | None = None) -> ctypes.CDLL:
    """Load (building first if needed) the oracle library and declare its prototypes."""
    global _lib
    if path is None:
        if _lib is not None:
            return _lib
        path = build()
    lib = ctypes.CDLL(path)
    sp = ctypes.POINTER(OrcShape)
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    up = ctypes.POINTER(ctypes.c_uint64)
    lib.orc_out_h.argtypes = [sp]
    lib.orc_out_h.restype = ctypes.c_int
    lib.orc_out_w.argtypes = [sp]
    lib.orc_out_w.restype = ctypes.c_int
    lib.orc_max_threads.argtypes = []
    lib.orc_max_threads.restype = ctypes.c_int
    lib.orc_set_threads.argtypes = [ctypes.c_int]
    lib.orc_set_threads.restype = None
    lib.orc_check_shape.argtypes = [sp]
    lib.orc_check_shape.restype = ctypes.c_int
    lib.orc_reconstruct.argtypes = [sp, fp, fp, fp, dp]
    lib.orc_reconstruct.restype = ctypes.c_uint64
    lib.orc_conv_dense.argtypes = [sp, fp, dp, dp]
    lib.orc_conv_dense.restype = ctypes.c_uint64
    lib.orc_stage1.argtypes = [sp, fp, fp, dp]
    lib.orc_stage1.restype = ctypes.c_uint64
    lib.orc_core.argtypes = [sp, dp, fp, dp]
    lib.orc_core.restype = ctypes.c_uint64
    lib.orc_stage3.argtypes = [sp, dp, fp, dp]
    lib.orc_stage3.restype = ctypes.c_uint64
    lib.orc_conv_factored.argtypes = [sp, fp, fp, fp, fp, dp, dp, dp, up]
    lib.orc_conv_factored.restype = ctypes.c_uint64
    if path == _LIB:
        _lib = lib
    return lib


def _f32(a, shape) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != tuple(shape):
        raise ValueError("expected array of shape %s, got %s" % (tuple(shape), a.shape))
    return a


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check(lib, sh: Shape):
    cs = sh.c_struct()
    rc = lib.orc_check_shape(ctypes.byref(cs))
    if rc != 0:
        raise ValueError("shape is not a computable layer: %r" % (sh,))
    return cs


def max_threads(lib=None) -> int:
    return (lib or load()).orc_max_threads()


def set_threads(n: int, lib=None) -> None:
    (lib or load()).orc_set_threads(int(n))


def reconstruct(sh: Shape, U_in, core, U_out, lib=None):
    """Eq. 1.  Returns (Wd float64 [C][N][K][K], MAC count)."""
    lib = lib or load()
    cs = _check(lib, sh)
    U_in = _f32(U_in, (sh.C, sh.R1))
    core = _f32(core, (sh.R1, sh.R2, sh.K, sh.K))
    U_out = _f32(U_out, (sh.R2, sh.N))
    Wd = np.empty((sh.C, sh.N, sh.K, sh.K), dtype=np.float64)
    macs = lib.orc_reconstruct(ctypes.byref(cs), _fptr(U_in), _fptr(core), _fptr(U_out), _dptr(Wd))
    return Wd, int(macs)


def conv_dense_with(sh: Shape, x, Wd, lib=None):
    """The definition, for a given dense kernel Wd[C][N][K][K] (float64)."""
    lib = lib or load()
    cs = _check(lib, sh)
    x = _f32(x, (sh.batch, sh.C, sh.H, sh.W))
    Wd = np.ascontiguousarray(Wd, dtype=np.float64)
    if Wd.shape != (sh.C, sh.N, sh.K, sh.K):
        raise ValueError("Wd has shape %s" % (Wd.shape,))
    y = np.empty((sh.batch, sh.N, sh.Ho, sh.Wo), dtype=np.float64)
    macs = lib.orc_conv_dense(ctypes.byref(cs), _fptr(x), _dptr(Wd), _dptr(y))
    return y, int(macs)


def conv_dense(sh: Shape, x, U_in, core, U_out, lib=None):
    """Eq. 1 followed by the definition of the convolution.  Returns (y float64, MACs of the conv)."""
    Wd, _ = reconstruct(sh, U_in, core, U_out, lib=lib)
    return conv_dense_with(sh, x, Wd, lib=lib)


def conv_factored(sh: Shape, x, U_in, core, U_out, lib=None, return_intermediates: bool = False):
    """Eqs. 2, 3, 4 in order.  Returns (y float64, [macs1, macs2, macs3]) and optionally z1, z2."""
    lib = lib or load()
    cs = _check(lib, sh)
    x = _f32(x, (sh.batch, sh.C, sh.H, sh.W))
    U_in = _f32(U_in, (sh.C, sh.R1))
    core = _f32(core, (sh.R1, sh.R2, sh.K, sh.K))
    U_out = _f32(U_out, (sh.R2, sh.N))
    z1 = np.empty((sh.batch, sh.R1, sh.H, sh.W), dtype=np.float64)
    z2 = np.empty((sh.batch, sh.R2, sh.Ho, sh.Wo), dtype=np.float64)
    y = np.empty((sh.batch, sh.N, sh.Ho, sh.Wo), dtype=np.float64)
    m3 = (ctypes.c_uint64 * 3)()
    lib.orc_conv_factored(ctypes.byref(cs), _fptr(x), _fptr(U_in), _fptr(core), _fptr(U_out),
                          _dptr(z1), _dptr(z2), _dptr(y), m3)
    macs = [int(m3[0]), int(m3[1]), int(m3[2])]
    if return_intermediates:
        return y, macs, z1, z2
    return y, macs


def apply_epilogue(y, bias=None, residual=None, relu: bool = False):
    """The output epilogue in float64: y + bias[n] + residual, then max(., 0) if relu.
    y: float64 [batch][N][Ho][Wo]; bias: [N] or None; residual: shaped like y or None."""
    out = np.array(y, dtype=np.float64, copy=True)
    if bias is not None:
        out += np.asarray(bias, dtype=np.float64).reshape(1, -1, 1, 1)
    if residual is not None:
        out += np.asarray(residual, dtype=np.float64)
    if relu:
        out = np.maximum(out, 0.0)
    return out
