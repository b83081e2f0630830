"""Thin Python binding over libtwist.so, the C-ABI library of the TwIST hot path on MI355X.

Only argument marshalling lives here: every step (sample, extract, forward+backward, optimizer step,
aggregate) runs inside the library's HIP kernels.  There is no CPU fallback: importing this package
without a built library raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
