"""libwcc: the forward path of the Wavelet Compressed Convolution layer
(Eq. WCC and the explicit algorithm in the appendix "Explicit WCC algorithm")
as hand-written HIP kernels for gfx950 behind a C ABI.

Sub-modules
-----------
``wcc``    thin ctypes binding over ``csrc/libwcc.so`` (argument marshalling only).
``synth``  seeded synthetic inputs (holds none of the method's arithmetic).

Nothing is imported eagerly so that ``synth`` can be used without the
compiled library being present.
"""

__all__ = ["wcc", "synth"]
