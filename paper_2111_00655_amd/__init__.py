"""MI355X-native fused-operator inference with placement search (C-ABI library
libcollage_mi.so plus this thin binding).  Build first:
    python -m paper_2111_00655_amd.build
"""
from .binding import *          # noqa: F401,F403
from .binding import ClgError, SYMBOLS, lib  # noqa: F401
from .runner import Session, Plan            # noqa: F401
