"""Builds libhashgrid.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.environ.get("HASHGRID_LIB") or os.path.join(_PKG, "libhashgrid.so")
PROBES_LIB_PATH = os.path.join(_PKG, "libhashgrid_probes.so")  # the benchmark's machine probes, a library of their own

SOURCES = ["hashgrid.hip", "bwd_binned.hip", "adam.hip", "loss.hip", "mlp_fused.hip", "mlp_bwd.hip"]
PROBE_SOURCES = ["probes.hip"]

# fp contraction is off so that the scale step of the encoding stays one rounded
# fp32 multiply (it decides voxel corners); FMAs are written out where wanted.
# Packed-fp32 instruction selection is disabled for this target.
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-munsafe-fp-atomics", "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


# Per-source flags.  mlp_bwd.hip: matrix-core results that the vector unit converts right away are kept
# out of the accumulation registers (a separate move per element otherwise).
SOURCE_FLAGS = {"mlp_bwd.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile_and_link(sources, out: str, verbose: bool, extra_flags) -> str:
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    tmp = out + f".tmp{os.getpid()}"
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="hashgrid_obj_") as objdir:
        def compile_one(src):
            obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc(), *flags, *SOURCE_FLAGS.get(src, []), *extra_flags, f"-I{INCLUDE}", f"-I{CSRC}", "-c", "-o", obj,
                   os.path.join(CSRC, src)]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        with ThreadPoolExecutor(max_workers=min(len(sources), os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, sources))
        link = [hipcc(), "--offload-arch=gfx950", "-fPIC", "-shared", "-o", tmp, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    os.replace(tmp, out)
    return out


def build_library(verbose: bool = False, extra_flags=(), out: str | None = None) -> str:
    """Compiles every source of libhashgrid (one hipcc process each, side by side) and links it."""
    return _compile_and_link(SOURCES, out or LIB_PATH, verbose, extra_flags)


def build_probes(verbose: bool = False, extra_flags=(), out: str | None = None) -> str:
    """libhashgrid_probes: the machine probes the benchmark uses for its measured denominators."""
    return _compile_and_link(PROBE_SOURCES, out or PROBES_LIB_PATH, verbose, extra_flags)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probes(verbose=True))
