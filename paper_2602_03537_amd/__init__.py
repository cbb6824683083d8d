"""MI355X-native Matryoshka-sliced quantized linear layers (libmq binding)."""
from .binding import *  # noqa: F401,F403
from . import binding as _binding

__all__ = list(_binding.__all__)
