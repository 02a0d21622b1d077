"""Multiresolution hash encoding for AMD MI355X: Python binding of the C-ABI
library (include/hashgrid.h).  `synth` holds the seeded synthetic workloads; the
probe_* functions bind the benchmark's machine probes (include/hashgrid_probes.h),
a library of their own."""
from .binding import (HG_F16, HG_F32, HG_INTERP_LINEAR, HG_INTERP_SMOOTHSTEP, HashGrid, HashGridError, LevelInfo,
                      adam_step, load_library, load_probes, loss_grad, mlp_bwd, mlp_fwd, probe_atomic_add, probe_copy, probe_gather,
                      probe_gather_lines, strerror)
from .model import HashGridModel

__all__ = ["HashGrid", "HashGridModel", "HashGridError", "LevelInfo", "adam_step", "loss_grad", "mlp_bwd", "mlp_fwd", "probe_copy", "probe_gather", "probe_atomic_add",
           "probe_gather_lines", "load_library", "load_probes", "strerror", "HG_F16", "HG_F32",
           "HG_INTERP_LINEAR", "HG_INTERP_SMOOTHSTEP"]
