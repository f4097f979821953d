"""MI355X-native decode hot path of the Louver KV-cache index: range query + sparse attention.

The work is done by hand-written HIP kernels in liblouver.so (sources under csrc/, C ABI in
include/louver.h); this package only marshals arguments.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LouverError, lib, lvr_config, lvr_stats, make_config  # noqa: F401
