"""FADE's batched probability step and arithmetic coder on one MI355X: thin ctypes binding of libfade.so.

Every function here only marshals arguments; all arithmetic of the path runs in the HIP kernels behind the
C ABI declared in include/fade.h. There is no CPU fallback: without the built library or without a GPU the
calls raise.
"""
from .binding import (BF16, F32, FROZEN, ONLINE_ADAM, TAPS, Config, Fade, FadeError, lib, make_config,  # noqa: F401
                      weights_nbytes)
from .buildlib import LIB, build  # noqa: F401

ONLINE_SUPPORTED = True
