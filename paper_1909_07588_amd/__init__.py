"""LAQ (lazily aggregated quantized gradients) hot path for MI355X.

Thin ctypes binding over liblaq_hip.so: argument marshalling only.  Every step
of the path runs in the library's HIP kernels; torch provides device memory
and the stream.  There is no CPU fallback: importing works without the
library (so the package can be inspected), but any call fails loudly.
"""
from .binding import (B_EXACT, MODE_FORCE_UPLOAD, Laq, LaqError, lib, lib_path,  # noqa: F401
                      p_stride, w_stride)
