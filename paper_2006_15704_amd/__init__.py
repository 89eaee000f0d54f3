"""MI355X-native bucketed gradient synchronization (the data-parallel hot path
of arXiv 2006.15704) behind a C-ABI library.  `binding` holds the ctypes
wrappers; `build` compiles the HIP sources with hipcc."""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
