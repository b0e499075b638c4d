"""Eigen Attention low-rank inference path for MI355X (gfx950): Python binding
over the C-ABI library libeigenattn.so built from csrc/ (see include/eigenattn.h)."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
