"""Convenience wrapper for callers that hold torch tensors: plan + packed weights + launch.

Marshalling only; the arithmetic is in libtdc.so.
"""
from __future__ import annotations

import ctypes
from typing import Optional

from . import binding as B


def _torch_stream(stream):
    """torch's stream object for None (the current stream), a raw stream handle, or a torch stream."""
    import torch
    if stream is None:
        return torch.cuda.current_stream()
    if isinstance(stream, int):
        return torch.cuda.ExternalStream(stream) if stream else torch.cuda.default_stream()
    return stream


def _order_after(conv, stream) -> None:
    """Make `stream` wait for conv's weight re-layout if that ran on another stream and may still be in flight.
    Nothing is enqueued on a stream that is being captured: finish the re-layout before capturing."""
    import torch
    ev = getattr(conv, "_pack_event", None)
    if ev is None or torch.cuda.is_current_stream_capturing():
        return
    if ev.query():                       # the re-layout is complete: no stream needs to wait any more
        conv._pack_event = None
        return
    ts = _torch_stream(stream)
    if ts.cuda_stream not in conv._ordered:
        ts.wait_event(ev)
        conv._ordered.add(ts.cuda_stream)


class TuckerConv2d:
    """One Tucker-2 convolution layer (paper section 3, Eqs. 2-4) bound to a device plan."""

    def __init__(self, layer, device: int = 0, tuning: Optional[B.tdc_tuning] = None, layout: int = B.LAYOUT_NCHW):
        """``layer`` has fields batch, C, N, H, W, R1, R2, K, stride, pad (e.g. workloads.Layer).
        ``layout``: LAYOUT_NCHW (x [B][C][H][W], y [B][N][Ho][Wo]) or LAYOUT_NHWC (x [B][H][W][C], y [B][Ho][Wo][N])."""
        self.shape = B.make_shape(layer.batch, layer.C, layer.N, layer.H, layer.W, layer.R1, layer.R2,
                                  layer.K, layer.stride, layer.pad, layout)
        self.Ho = B.tdc_out_size(layer.H, layer.K, layer.stride, layer.pad)
        self.Wo = B.tdc_out_size(layer.W, layer.K, layer.stride, layer.pad)
        self.plan = B.tdc_plan_create(self.shape, device, tuning)
        self.device = device
        self._weights = None

    def out_shape(self):
        """Shape of y in the plan's layout."""
        s = self.shape
        return (s.batch, self.Ho, self.Wo, s.N) if s.layout == B.LAYOUT_NHWC else (s.batch, s.N, self.Ho, self.Wo)

    def describe(self) -> str:
        return B.tdc_plan_describe(self.plan)

    def tuning(self) -> dict:
        return B.tdc_plan_get_tuning(self.plan).as_dict()

    def kernel_count(self) -> int:
        return B.tdc_plan_kernel_count(self.plan)

    def pack(self, U_in, core, U_out, stream=None) -> None:
        """Re-lay the weights out once; the tensors must stay alive and unchanged.

        The re-layout runs on ``stream`` (default: the current stream).  The library orders nothing between streams,
        so a later call or bind() on another stream is made to wait for it here (an event recorded now)."""
        self._weights = (U_in, core, U_out)
        B.tdc_plan_pack_weights(self.plan, U_in, core, U_out, stream)
        ts = _torch_stream(stream)
        self._pack_event = ts.record_event()
        self._ordered = {ts.cuda_stream}

    def _order_after_pack(self, stream) -> None:
        _order_after(self, stream)

    def __call__(self, x, y=None, weights=None, stream=None, bias=None, residual=None, relu=False):
        """y = layer(x), optionally followed by the fused epilogue y = relu?(y + bias[n] + residual)."""
        import torch
        U_in, core, U_out = weights if weights is not None else self._weights
        self._order_after_pack(stream)
        if y is None:
            y = torch.empty(self.out_shape(), device=x.device, dtype=torch.float32)
        if bias is None and residual is None and not relu:
            B.tdc_conv_tucker2(self.plan, x, U_in, core, U_out, y, self.shape, stream)
        else:
            B.tdc_conv_tucker2_ex(self.plan, x, U_in, core, U_out, y, self.shape,
                                  B.make_epilogue(bias, residual, relu), stream)
        return y

    def bind(self, x, y, weights=None, stream=None, bias=None, residual=None, relu=False):
        """Marshal the arguments of tdc_conv_tucker2(_ex) once and return a zero-argument launcher.

        For callers that enqueue the same buffers repeatedly: the per-call cost is one foreign
        call.  The tensors and the stream must outlive the launcher."""
        U_in, core, U_out = weights if weights is not None else self._weights
        self._order_after_pack(stream)
        vp = ctypes.c_void_p
        args = (self.plan, vp(B._stream(stream)), vp(x.data_ptr()), vp(U_in.data_ptr()), vp(core.data_ptr()),
                vp(U_out.data_ptr()), vp(y.data_ptr()), ctypes.byref(self.shape))
        if bias is None and residual is None and not relu:
            fn = B.load().tdc_conv_tucker2
        else:
            fn = B.load().tdc_conv_tucker2_ex
            epi = B.make_epilogue(bias, residual, relu)
            args = args + (ctypes.byref(epi),)

        def launch():
            rc = fn(*args)
            if rc:
                raise B.TdcError(rc, "tdc_conv_tucker2")

        return launch

    def close(self) -> None:
        if self.plan is not None:
            B.tdc_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DenseConv2d:
    """The undecomposed K x K layer with the kernel W[C][N][K][K] of Eq. 1, on the same library: the
    "original convolution" the rank-selection threshold test (paper section 6) compares against."""

    def __init__(self, layer, device: int = 0, tuning: Optional[B.tdc_tuning] = None, layout: int = B.LAYOUT_NCHW):
        self.shape = B.make_shape(layer.batch, layer.C, layer.N, layer.H, layer.W, layer.R1, layer.R2,
                                  layer.K, layer.stride, layer.pad, layout)
        self.Ho = B.tdc_out_size(layer.H, layer.K, layer.stride, layer.pad)
        self.Wo = B.tdc_out_size(layer.W, layer.K, layer.stride, layer.pad)
        t = tuning if tuning is not None else B.make_tuning()
        t.variant = B.VARIANT_DENSE
        self.plan = B.tdc_plan_create(self.shape, device, t)
        self.device = device
        self._W = None

    def out_shape(self):
        """Shape of y in the plan's layout."""
        s = self.shape
        return (s.batch, self.Ho, self.Wo, s.N) if s.layout == B.LAYOUT_NHWC else (s.batch, s.N, self.Ho, self.Wo)

    def describe(self) -> str:
        return B.tdc_plan_describe(self.plan)

    def tuning(self) -> dict:
        return B.tdc_plan_get_tuning(self.plan).as_dict()

    def pack(self, W, stream=None) -> None:
        self._W = W
        B.tdc_plan_pack_dense(self.plan, W, stream)
        ts = _torch_stream(stream)
        self._pack_event = ts.record_event()
        self._ordered = {ts.cuda_stream}

    def __call__(self, x, y=None, W=None, stream=None, bias=None, residual=None, relu=False):
        import torch
        W = W if W is not None else self._W
        _order_after(self, stream)
        if y is None:
            y = torch.empty(self.out_shape(), device=x.device, dtype=torch.float32)
        if bias is None and residual is None and not relu:
            B.tdc_conv_dense(self.plan, x, W, y, self.shape, stream)
        else:
            B.tdc_conv_dense_ex(self.plan, x, W, y, self.shape, B.make_epilogue(bias, residual, relu), stream)
        return y

    def bind(self, x, y, W=None, stream=None, bias=None, residual=None, relu=False):
        """Zero-argument launcher with the arguments of tdc_conv_dense(_ex) marshalled once."""
        W = W if W is not None else self._W
        _order_after(self, stream)
        vp = ctypes.c_void_p
        args = (self.plan, vp(B._stream(stream)), vp(x.data_ptr()), vp(W.data_ptr()), vp(y.data_ptr()),
                ctypes.byref(self.shape))
        if bias is None and residual is None and not relu:
            fn = B.load().tdc_conv_dense
        else:
            fn = B.load().tdc_conv_dense_ex
            epi = B.make_epilogue(bias, residual, relu)
            args = args + (ctypes.byref(epi),)

        def launch():
            rc = fn(*args)
            if rc:
                raise B.TdcError(rc, "tdc_conv_dense")

        return launch

    def close(self) -> None:
        if self.plan is not None:
            B.tdc_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
