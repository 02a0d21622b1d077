"""Multiresolution hash encoding for AMD MI355X: Python binding of the C-ABI
library (include/hashgrid.h).  `synth` holds the seeded synthetic workloads."""
from .binding import (HG_F16, HG_F32, HG_INTERP_LINEAR, HG_INTERP_SMOOTHSTEP, HashGrid, HashGridError, LevelInfo,
                      adam_step, load_library, probe_atomic_add, probe_copy, probe_gather, strerror)

__all__ = ["HashGrid", "HashGridError", "LevelInfo", "adam_step", "probe_copy", "probe_gather", "probe_atomic_add", "load_library", "strerror", "HG_F16", "HG_F32",
           "HG_INTERP_LINEAR", "HG_INTERP_SMOOTHSTEP"]
