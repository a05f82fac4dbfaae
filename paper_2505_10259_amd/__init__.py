"""MI355X-native speculative draft/verify hot path (C-ABI library + thin ctypes binding).

``from paper_2505_10259_amd import binding`` loads libspecverify.so (building it with hipcc if it
is missing) and exposes the functions of include/specverify.h under the same names.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
from .harness import Session  # noqa: F401
