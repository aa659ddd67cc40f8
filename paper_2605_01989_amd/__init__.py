"""MI355X-native receiver-side bounded-loss gradient aggregation (DBLP).

Thin Python binding over the C-ABI library libdblp_agg.so (hand-written HIP
kernels for gfx950).  Argument marshalling only: every step of the path runs
in the library's kernels.  There is no CPU fallback; a missing library is an
error.
"""
from .binding import (Aggregator, ClrController, DblpError, lib, policy_linear, policy_three_level,  # noqa: F401
                      policy_two_level, sumsq_static)
