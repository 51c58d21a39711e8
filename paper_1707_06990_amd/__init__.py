"""Memory-efficient DenseNet dense block for AMD MI355X: C-ABI library + thin binding."""
from .binding import *  # noqa: F401,F403
from . import binding as _binding

EXPORTED = _binding.EXPORTED
