"""MI355X-native Stochastic Gradient Push update (arXiv 1811.10792).

csrc/ holds the HIP kernels and the C ABI of include/sgp.h; binding.py marshals
arguments; synthetic.py draws the seeded benchmark inputs.  Importing the package loads nothing;
the HIP library is loaded on first use and its absence is an error.
"""
from .binding import (SGP, SgpError, Stats, load_library, sgp_consensus_stats_noalloc, sgp_copy,  # noqa: F401
                      sgp_schedule, sgp_stream_pattern, status_string)

__all__ = ["SGP", "SgpError", "Stats", "load_library", "sgp_consensus_stats_noalloc", "sgp_copy", "sgp_schedule",
           "sgp_stream_pattern", "status_string"]
