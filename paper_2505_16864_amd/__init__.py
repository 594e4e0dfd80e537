"""MI355X-native attention carving (block-sparse attention over curve-ordered video tokens).

The package is a thin binding of libjenga.so; see include/jenga.h for the contract.
"""
from .binding import *  # noqa: F401,F403
from .binding import (jenga_config, jenga_plan_info_t, JengaError, make_config, EXPORTS, raw)  # noqa: F401
