"""Thin ctypes binding of libtdc.so, with the same names as ``include/tdc.h``.

Argument marshalling only: every step of the layer runs in the library's HIP
kernels.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the built library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libtdc.so")

TDC_OK = 0
TDC_ERR_NULL = -1
TDC_ERR_BAD_SHAPE = -2
TDC_ERR_SHAPE_MISMATCH = -3
TDC_ERR_UNSUPPORTED = -4
TDC_ERR_ALLOC = -5
TDC_ERR_HIP = -6
TDC_ERR_BAD_TUNING = -7
TDC_ERR_TOO_LARGE = -8
TDC_ERR_NO_CONVERGENCE = -9
STATIC_SCRATCH_BYTES = 32 * 1024 * 1024

LAYOUT_NCHW, LAYOUT_NHWC = 0, 1
VARIANT_AUTO, VARIANT_NAIVE, VARIANT_SPLIT, VARIANT_FUSED, VARIANT_CHAIN, VARIANT_DENSE, VARIANT_MERGED = 0, 1, 2, 3, 4, 5, 6
VARIANT_FUSED_MERGED = 7
VARIANT_MERGED_XCD = 8
VARIANT_NAMES = {0: "auto", 1: "naive", 2: "split", 3: "fused", 4: "chain", 5: "dense", 6: "merged", 7: "fused_merged",
                 8: "merged_xcd"}
ERR_WAIT = -10

# every symbol include/tdc.h declares
EXPORTS = ["tdc_plan_create", "tdc_plan_create_tuned", "tdc_plan_pack_weights", "tdc_conv_tucker2",
           "tdc_plan_destroy", "tdc_plan_get_tuning", "tdc_plan_describe", "tdc_plan_workspace_bytes",
           "tdc_plan_kernel_count", "tdc_status_string", "tdc_version", "tdc_out_size",
           "tdc_select_tuning", "tdc_launch_null", "tdc_plan_pack_dense", "tdc_conv_dense", "tdc_select_ranks",
           "tdc_conv_tucker2_ex", "tdc_conv_dense_ex", "tdc_hosvd_tucker2", "tdc_admm_project",
           "tdc_conv_tucker2_static", "tdc_model_terms", "tdc_plan_status", "tdc_plan_set_wait_limit", "tdc_plan_waits_given_up"]


class tdc_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("batch", "C", "N", "H", "W", "R1", "R2", "K", "stride", "pad", "layout")]


class tdc_tuning(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("tile_h", ctypes.c_int32), ("tile_w", ctypes.c_int32),
                ("waves", ctypes.c_int32 * 3), ("mb", ctypes.c_int32 * 3), ("pb", ctypes.c_int32 * 3)]

    def as_dict(self):
        return {"variant": VARIANT_NAMES.get(self.variant, self.variant), "tile_h": self.tile_h,
                "tile_w": self.tile_w, "waves": list(self.waves), "mb": list(self.mb), "pb": list(self.pb)}


class tdc_rank_entry(ctypes.Structure):
    _fields_ = [("R1", ctypes.c_int32), ("R2", ctypes.c_int32), ("latency_us", ctypes.c_double)]


class tdc_rank_layer(ctypes.Structure):
    _fields_ = [("shape", tdc_shape), ("table", ctypes.POINTER(tdc_rank_entry)), ("n_entries", ctypes.c_int32),
                ("dense_latency_us", ctypes.c_double)]


class tdc_rank_choice(ctypes.Structure):
    _fields_ = [("decomposed", ctypes.c_int32), ("R1", ctypes.c_int32), ("R2", ctypes.c_int32),
                ("latency_us", ctypes.c_double), ("macs", ctypes.c_double)]


class tdc_epilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("residual", ctypes.c_void_p), ("relu", ctypes.c_int32)]


class TdcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, status_string(status)))


_lib = None


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libtdc.so and declare prototypes.  Raises if the library has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError("%s is missing: build it first (python -m paper_2211_03715_amd.build); "
                           "there is no CPU fallback" % p)
    lib = ctypes.CDLL(p)
    vp, ip = ctypes.c_void_p, ctypes.c_int
    sp, tp = ctypes.POINTER(tdc_shape), ctypes.POINTER(tdc_tuning)
    lib.tdc_plan_create.argtypes = [ctypes.POINTER(vp), sp, ip]
    lib.tdc_plan_create.restype = ip
    lib.tdc_plan_create_tuned.argtypes = [ctypes.POINTER(vp), sp, ip, tp]
    lib.tdc_plan_create_tuned.restype = ip
    lib.tdc_plan_pack_weights.argtypes = [vp, vp, vp, vp, vp]
    lib.tdc_plan_pack_weights.restype = ip
    lib.tdc_conv_tucker2.argtypes = [vp, vp, vp, vp, vp, vp, vp, sp]
    lib.tdc_conv_tucker2.restype = ip
    lib.tdc_conv_tucker2_static.argtypes = [vp, vp, vp, vp, vp, vp, sp]
    lib.tdc_conv_tucker2_static.restype = ip
    lib.tdc_plan_pack_dense.argtypes = [vp, vp, vp]
    lib.tdc_plan_pack_dense.restype = ip
    lib.tdc_conv_dense.argtypes = [vp, vp, vp, vp, vp, sp]
    lib.tdc_conv_dense.restype = ip
    ep = ctypes.POINTER(tdc_epilogue)
    lib.tdc_conv_tucker2_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, sp, ep]
    lib.tdc_conv_tucker2_ex.restype = ip
    lib.tdc_conv_dense_ex.argtypes = [vp, vp, vp, vp, vp, sp, ep]
    lib.tdc_conv_dense_ex.restype = ip
    lib.tdc_plan_destroy.argtypes = [vp]
    lib.tdc_plan_destroy.restype = ip
    lib.tdc_plan_get_tuning.argtypes = [vp, tp]
    lib.tdc_plan_get_tuning.restype = ip
    lib.tdc_plan_describe.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t]
    lib.tdc_plan_describe.restype = ip
    lib.tdc_plan_workspace_bytes.argtypes = [vp]
    lib.tdc_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.tdc_plan_kernel_count.argtypes = [vp]
    lib.tdc_plan_kernel_count.restype = ip
    lib.tdc_status_string.argtypes = [ip]
    lib.tdc_status_string.restype = ctypes.c_char_p
    lib.tdc_version.argtypes = []
    lib.tdc_version.restype = ip
    lib.tdc_out_size.argtypes = [ip, ip, ip, ip]
    lib.tdc_out_size.restype = ip
    lib.tdc_select_tuning.argtypes = [sp, ip, ip, tp]
    lib.tdc_select_tuning.restype = ip
    lib.tdc_model_terms.argtypes = [sp, tp, ip, ip, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_char_p), ip,
                                    ctypes.POINTER(ip), ctypes.POINTER(ctypes.c_char_p)]
    lib.tdc_model_terms.restype = ip
    lib.tdc_launch_null.argtypes = [vp]
    lib.tdc_launch_null.restype = ip
    lib.tdc_plan_status.argtypes = [vp]
    lib.tdc_plan_status.restype = ip
    lib.tdc_plan_set_wait_limit.argtypes = [vp, ctypes.c_uint]
    lib.tdc_plan_set_wait_limit.restype = ip
    lib.tdc_plan_waits_given_up.argtypes = [vp, ctypes.POINTER(ctypes.c_uint)]
    lib.tdc_plan_waits_given_up.restype = ip
    lib.tdc_select_ranks.argtypes = [ctypes.POINTER(tdc_rank_layer), ip, ctypes.c_double, ctypes.c_double,
                                     ctypes.c_double, ctypes.POINTER(tdc_rank_choice)]
    lib.tdc_select_ranks.restype = ip
    fp = ctypes.POINTER(ctypes.c_float)
    lib.tdc_hosvd_tucker2.argtypes = [fp, ip, ip, ip, ip, ip, fp, fp, fp]
    lib.tdc_hosvd_tucker2.restype = ip
    lib.tdc_admm_project.argtypes = [fp, fp, ip, ip, ip, ip, ip, fp]
    lib.tdc_admm_project.restype = ip
    if path is None:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().tdc_status_string(int(status)).decode()


tdc_status_string = status_string


def tdc_version() -> int:
    return load().tdc_version()


def tdc_out_size(n: int, K: int, stride: int, pad: int) -> int:
    return load().tdc_out_size(n, K, stride, pad)


def make_shape(batch, C, N, H, W, R1, R2, K=3, stride=1, pad=1, layout=0) -> tdc_shape:
    return tdc_shape(batch, C, N, H, W, R1, R2, K, stride, pad, layout)


def make_tuning(variant=0, tile_h=0, tile_w=0, waves=(0, 0, 0), mb=(0, 0, 0), pb=(0, 0, 0)) -> tdc_tuning:
    t = tdc_tuning()
    t.variant, t.tile_h, t.tile_w = variant, tile_h, tile_w
    for i in range(3):
        t.waves[i], t.mb[i], t.pb[i] = waves[i], mb[i], pb[i]
    return t


def tdc_select_tuning(shape: tdc_shape, compute_units: int = 256, lds_bytes: int = 160 * 1024,
                      tuning: Optional[tdc_tuning] = None) -> tdc_tuning:
    t = tuning if tuning is not None else tdc_tuning()
    rc = load().tdc_select_tuning(ctypes.byref(shape), compute_units, lds_bytes, ctypes.byref(t))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_select_tuning")
    return t


def tdc_model_terms(shape: tdc_shape, tuning: tdc_tuning, compute_units: int = 256, lds_bytes: int = 160 * 1024):
    """(model name, term names, terms) of the selector's estimate for a fully specified tuning."""
    terms = (ctypes.c_double * 32)()
    names = (ctypes.c_char_p * 32)()
    n, model = ctypes.c_int(0), ctypes.c_char_p()
    rc = load().tdc_model_terms(ctypes.byref(shape), ctypes.byref(tuning), compute_units, lds_bytes, terms, names, 32,
                                ctypes.byref(n), ctypes.byref(model))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_model_terms")
    return model.value.decode(), [names[i].decode() for i in range(n.value)], [terms[i] for i in range(n.value)]


def tdc_plan_create(shape: tdc_shape, device: int = 0, tuning: Optional[tdc_tuning] = None) -> ctypes.c_void_p:
    lib = load()
    plan = ctypes.c_void_p()
    if tuning is None:
        rc = lib.tdc_plan_create(ctypes.byref(plan), ctypes.byref(shape), device)
    else:
        rc = lib.tdc_plan_create_tuned(ctypes.byref(plan), ctypes.byref(shape), device, ctypes.byref(tuning))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_create")
    return plan


def tdc_plan_create_tuned(shape: tdc_shape, device: int, tuning: tdc_tuning) -> ctypes.c_void_p:
    return tdc_plan_create(shape, device, tuning)


def tdc_plan_destroy(plan) -> None:
    rc = load().tdc_plan_destroy(plan)
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_destroy")


def _ptr(t):
    """Device pointer of a torch tensor (or pass an int / None through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def tdc_plan_pack_weights(plan, U_in, core, U_out, stream=None) -> None:
    rc = load().tdc_plan_pack_weights(plan, _stream(stream), _ptr(U_in), _ptr(core), _ptr(U_out))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_pack_weights")


def tdc_conv_tucker2(plan, x, U_in, core, U_out, y, shape: tdc_shape, stream=None) -> None:
    rc = load().tdc_conv_tucker2(plan, _stream(stream), _ptr(x), _ptr(U_in), _ptr(core), _ptr(U_out),
                                 _ptr(y), ctypes.byref(shape))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_conv_tucker2")


def tdc_conv_tucker2_static(x, U_in, core, U_out, y, shape: tdc_shape, stream=None) -> None:
    """The plan-less call that allocates nothing (scratch in a static device array of the library)."""
    rc = load().tdc_conv_tucker2_static(_stream(stream), _ptr(x), _ptr(U_in), _ptr(core), _ptr(U_out), _ptr(y),
                                        ctypes.byref(shape))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_conv_tucker2_static")


def tdc_plan_pack_dense(plan, W, stream=None) -> None:
    rc = load().tdc_plan_pack_dense(plan, _stream(stream), _ptr(W))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_pack_dense")


def tdc_conv_dense(plan, x, W, y, shape: tdc_shape, stream=None) -> None:
    rc = load().tdc_conv_dense(plan, _stream(stream), _ptr(x), _ptr(W), _ptr(y), ctypes.byref(shape))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_conv_dense")


def make_epilogue(bias=None, residual=None, relu=False) -> tdc_epilogue:
    """bias / residual: torch tensors on the plan's device (or raw device pointers) or None."""
    return tdc_epilogue(_ptr(bias), _ptr(residual), 1 if relu else 0)


def tdc_conv_tucker2_ex(plan, x, U_in, core, U_out, y, shape: tdc_shape, epilogue: Optional[tdc_epilogue], stream=None) -> None:
    rc = load().tdc_conv_tucker2_ex(plan, _stream(stream), _ptr(x), _ptr(U_in), _ptr(core), _ptr(U_out), _ptr(y),
                                    ctypes.byref(shape), ctypes.byref(epilogue) if epilogue is not None else None)
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_conv_tucker2_ex")


def tdc_conv_dense_ex(plan, x, W, y, shape: tdc_shape, epilogue: Optional[tdc_epilogue], stream=None) -> None:
    rc = load().tdc_conv_dense_ex(plan, _stream(stream), _ptr(x), _ptr(W), _ptr(y), ctypes.byref(shape),
                                  ctypes.byref(epilogue) if epilogue is not None else None)
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_conv_dense_ex")


def tdc_plan_get_tuning(plan) -> tdc_tuning:
    t = tdc_tuning()
    rc = load().tdc_plan_get_tuning(plan, ctypes.byref(t))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_get_tuning")
    return t


def tdc_plan_describe(plan) -> str:
    buf = ctypes.create_string_buffer(512)
    rc = load().tdc_plan_describe(plan, buf, 512)
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_describe")
    return buf.value.decode()


def tdc_plan_workspace_bytes(plan) -> int:
    return int(load().tdc_plan_workspace_bytes(plan))


def tdc_plan_kernel_count(plan) -> int:
    return int(load().tdc_plan_kernel_count(plan))


def tdc_plan_status(plan) -> int:
    """TDC_OK, or ERR_WAIT once a kernel of a MERGED_XCD plan has reported that it cannot run here (read after synchronising)."""
    return int(load().tdc_plan_status(plan))


def tdc_plan_set_wait_limit(plan, polls: int) -> None:
    rc = load().tdc_plan_set_wait_limit(plan, polls)
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_set_wait_limit")


def tdc_plan_waits_given_up(plan) -> int:
    n = ctypes.c_uint(0)
    rc = load().tdc_plan_waits_given_up(plan, ctypes.byref(n))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_plan_waits_given_up")
    return int(n.value)


def tdc_launch_null(stream=None) -> None:
    rc = load().tdc_launch_null(_stream(stream))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_launch_null")


def tdc_select_ranks(layers, tables, dense_latency, budget: float, theta: float = 0.15, tie_tol: float = 0.0):
    """``layers``: objects or dicts with batch, C, N, H, W, K, stride, pad; ``tables``: per layer a list of
    (R1, R2, latency_us); ``dense_latency``: per layer the original convolution's latency.
    Returns one dict per layer: decomposed, R1, R2, latency_us, macs."""
    n = len(layers)
    if not (n == len(tables) == len(dense_latency)):
        raise ValueError("layers, tables and dense_latency must have the same length")
    arr = (tdc_rank_layer * n)()
    keep = []
    for i, (L, tab, t2) in enumerate(zip(layers, tables, dense_latency)):
        g = (lambda k: L[k]) if isinstance(L, dict) else (lambda k: getattr(L, k))
        arr[i].shape = make_shape(g("batch"), g("C"), g("N"), g("H"), g("W"), 1, 1, g("K"), g("stride"), g("pad"))
        ent = (tdc_rank_entry * max(1, len(tab)))()
        for j, (r1, r2, t) in enumerate(tab):
            ent[j].R1, ent[j].R2, ent[j].latency_us = int(r1), int(r2), float(t)
        keep.append(ent)
        arr[i].table = ctypes.cast(ent, ctypes.POINTER(tdc_rank_entry))
        arr[i].n_entries = len(tab)
        arr[i].dense_latency_us = float(t2)
    out = (tdc_rank_choice * n)()
    rc = load().tdc_select_ranks(arr, n, float(budget), float(theta), float(tie_tol), out)
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_select_ranks")
    return [{"decomposed": bool(o.decomposed), "R1": o.R1, "R2": o.R2, "latency_us": o.latency_us, "macs": o.macs}
            for o in out]


def _host_f32(a, shape=None):
    import numpy as np
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and a.shape != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a


def tdc_hosvd_tucker2(W, R1: int, R2: int):
    """W: numpy float32 [C][N][K][K] on the host.  Returns (U_in [C][R1], core [R1][R2][K][K], U_out [R2][N])."""
    import numpy as np
    W = _host_f32(W)
    if W.ndim != 4 or W.shape[2] != W.shape[3]:
        raise ValueError("W must be [C][N][K][K]")
    C, N, K, _ = W.shape
    U_in = np.empty((C, max(R1, 1)), dtype=np.float32)
    core = np.empty((max(R1, 1), max(R2, 1), K, K), dtype=np.float32)
    U_out = np.empty((max(R2, 1), N), dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    rc = load().tdc_hosvd_tucker2(W.ctypes.data_as(fp), C, N, K, R1, R2, U_in.ctypes.data_as(fp), core.ctypes.data_as(fp),
                                  U_out.ctypes.data_as(fp))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_hosvd_tucker2")
    return U_in, core, U_out


def tdc_admm_project(K_weights, M, R1: int, R2: int):
    """K_hat <- proj(K + M), M <- M + K - K_hat.  numpy float32 [C][N][K][K] on the host; returns (K_hat, M_new)."""
    import numpy as np
    Kw = _host_f32(K_weights)
    Mn = _host_f32(M, Kw.shape).copy()
    C, N, K, _ = Kw.shape
    K_hat = np.empty_like(Kw)
    fp = ctypes.POINTER(ctypes.c_float)
    rc = load().tdc_admm_project(Kw.ctypes.data_as(fp), Mn.ctypes.data_as(fp), C, N, K, R1, R2, K_hat.ctypes.data_as(fp))
    if rc != TDC_OK:
        raise TdcError(rc, "tdc_admm_project")
    return K_hat, Mn
