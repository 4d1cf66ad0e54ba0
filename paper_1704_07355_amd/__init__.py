"""Quick ADC hot path for AMD MI355X: ctypes binding over the C-ABI HIP library."""

from .binding import *  # noqa: F401,F403
from .binding import lib, QadcError, EXPORTS  # noqa: F401
