"""MI355X-native BAOC gradient-stream profiler and allocator (thin binding over libbaoc.so)."""
from .binding import (BaocError, BlockStats, Config, ProfileParams, Profiler, RiskParams, Sampler, allocate, partition,
                      load_library, status_string, STAT_FIELDS)

__all__ = ["BaocError", "BlockStats", "Config", "ProfileParams", "Profiler", "RiskParams", "Sampler", "allocate", "partition",
           "load_library", "status_string", "STAT_FIELDS"]
