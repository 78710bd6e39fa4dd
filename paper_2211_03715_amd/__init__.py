"""MI355X-native inference of a Tucker-2-format convolution layer (paper section 3, Eqs. 1-4).

``workloads`` names the synthetic layer shapes and draws seeded inputs;
``binding`` is the thin ctypes layer over the C-ABI library ``libtdc.so``
(HIP kernels for gfx950).  Nothing here falls back to a CPU implementation:
calling the binding without the built library raises.
"""
