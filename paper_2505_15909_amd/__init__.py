"""MI355X-native RTN weight-only quantised linear layers (arXiv 2505.15909).

Everything computes in the HIP library behind include/rtn.h; see binding.py.
"""
from .binding import *  # noqa: F401,F403
from .binding import RtnError, LayerPlan, rtn_linear_cfg, EXPORTS, _lib  # noqa: F401
