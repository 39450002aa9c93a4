"""MI355X-native mixed-precision (int8 / int16 / fp16) conv, FC and mixture-of-experts inference
kernels behind a C ABI (include/mpq.h), with a thin ctypes binding."""
from . import binding  # noqa: F401
