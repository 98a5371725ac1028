"""QuantCache's quantized-linear hot path for one MI355X: libqc.so (HIP, gfx950) + a ctypes binding."""
from . import binding  # noqa: F401  (loading the shared library itself is deferred to first use)
