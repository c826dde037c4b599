"""MI355X-native intra-kernel region profiler: thin Python binding over libkperf.so.

Every step of the hot path runs in the HIP library; this package only marshals
arguments (torch tensors give device pointers and streams).  There is no CPU
fallback: importing `binding` without a built libkperf.so raises.
"""
from .binding import *  # noqa: F401,F403
