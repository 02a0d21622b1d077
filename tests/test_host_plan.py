"""The plan of the sorted backward pass, checked on the host, point by point (no GPU): tests/plan_check.hip
is compiled for the host and runs the same rows_of the count and scatter kernels run.  For every pair
of corners it must give the bin, the chunk-local index and the step to the upper corner that lead,
under the record's rules, to the two entries Section 3 and Eq. 4 define, within the bounds the
kernels index with (bin inside its level, index inside its chunk, chunk inside 4096 entries)."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from paper_2201_05989_amd import binding, synth
from paper_2201_05989_amd.build import CSRC, INCLUDE, LIB_PATH, hipcc

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def plan_check(tmp_path_factory):
    binding.load_library()  # raises if libhashgrid.so is not built
    out = str(tmp_path_factory.mktemp("plan") / "libplan_check.so")
    lib_dir = os.path.dirname(LIB_PATH)
    cmd = [hipcc(), "--cuda-host-only", "-O2", "-ffp-contract=off", "-fPIC", "-shared", f"-I{INCLUDE}", f"-I{CSRC}",
           os.path.join(HERE, "plan_check.hip"), "-o", out, f"-L{lib_dir}", "-lhashgrid", f"-Wl,-rpath,{lib_dir}"]
    subprocess.run(cmd, check=True, capture_output=True)
    lib = ctypes.CDLL(out)
    lib.plan_check.restype = ctypes.c_uint64
    lib.plan_check.argtypes = [ctypes.POINTER(binding.hashgrid_config), ctypes.c_uint32, ctypes.c_void_p,
                               ctypes.POINTER(ctypes.c_uint64)]

    def run(d, L, F, T, N_min, N_max, interp, x):
        cfg = binding.hashgrid_config(d, L, F, T, N_min, N_max, binding.HG_F16, binding.HG_F16, interp, binding.HG_F32)
        x = np.ascontiguousarray(x, dtype=np.float32)
        crossing = ctypes.c_uint64(0)
        bad = lib.plan_check(ctypes.byref(cfg), len(x), x.ctypes.data, ctypes.byref(crossing))
        return bad, crossing.value

    run.lib = lib
    return run


@pytest.mark.parametrize("name", ["tiny2d", "image2d", "sdf3d", "nerf3d", "large3d"])
def test_plan_of_every_workload(plan_check, name):
    w = synth.WORKLOADS[name]
    x = synth.make_points(w.points, np.random.default_rng(11), 20000, w.d)
    for interp in (0, 1):
        bad, crossing = plan_check(w.d, w.L, w.F, w.T, w.N_min, w.N_max, interp, x)
        assert bad == 0
        assert (crossing > 0) == (w.N_max >= 4096)  # pairs straddle chunks only at such resolutions


@pytest.mark.parametrize("seed", range(40))
def test_plan_of_random_configurations(plan_check, seed):
    rng = np.random.default_rng(300 + seed)
    d = int(rng.integers(2, 4))
    F = int(rng.choice([1, 2, 4, 8]))
    L = int(rng.integers(1, 17))
    T = 1 << int(rng.integers(0, 24 if F == 8 else 25))
    N_min = int(rng.integers(1, 40))
    N_max = int(N_min * rng.choice([1, 2, 7, 100, 3000]) + rng.integers(0, 5))
    interp = int(rng.integers(0, 2))
    x = synth.points_uniform(rng, 3000, d)
    # grid vertices, the last voxel and the voxels whose pair straddles two chunks, on top of random points
    x[:50] = 0.0
    x[50:100] = 1 - 2.0 ** -24
    x[100:400, 0] = ((4095.75 + 4096.0 * rng.integers(0, 2, 300)) / 8192.0).astype(np.float32)
    bad, _ = plan_check(d, L, F, T, N_min, N_max, interp, x)
    served = binding.HashGrid(d, L, F, T, N_min, N_max, "f16", "f16", interp).bwd_workspace_bytes(3000) > 0
    assert bad == (0 if served else 2 ** 64 - 1)


@pytest.mark.parametrize("seed", range(24))
def test_plan_with_a_record_per_corner(plan_check, seed):
    # table sizes that are not powers of two (Eq. 4's mod T) and one-dimensional inputs: no pairing
    rng = np.random.default_rng(700 + seed)
    d = int(rng.integers(1, 4))
    F = int(rng.choice([1, 2, 4, 8]))
    L = int(rng.integers(1, 12))
    T = int(rng.choice([1, 2, 3, 1000, 4097, 12345, 1000003, 5 * 2 ** 20 + 1])) if d > 1 or seed % 2 else 1 << int(rng.integers(0, 22))
    N_min = int(rng.integers(1, 40))
    N_max = int(N_min * rng.choice([1, 2, 7, 100, 3000]) + rng.integers(0, 5))
    interp = int(rng.integers(0, 2))
    x = synth.points_uniform(rng, 3000, d)
    x[:50] = 0.0
    x[50:100] = 1 - 2.0 ** -24
    bad, _ = plan_check(d, L, F, T, N_min, N_max, interp, x)
    served = binding.HashGrid(d, L, F, T, N_min, N_max, "f16", "f16", interp).bwd_workspace_bytes(3000) > 0
    assert served and bad == 0


def test_plan_where_half_of_the_pairs_straddle_two_chunks(plan_check):
    rng = np.random.default_rng(5)
    for d in (2, 3):
        x = synth.points_uniform(rng, 6000, d)
        x[:3000, 0] = ((4095.75 + 4096.0 * rng.integers(0, 2, 3000)) / 8192.0).astype(np.float32)
        bad, crossing = plan_check(d, 3, 2, 1 << 16, 8192, 32768, 0, x)
        assert bad == 0 and crossing >= 3 * 3000


def test_order_of_records_inside_a_run_is_a_permutation(plan_check):
    """The scatter pass spreads the records a tile puts into one bin (records of neighbouring points apart,
    for the accumulate pass's LDS atomics): whatever the run length, every slot of the run is used exactly once."""
    plan_check.lib.spread_check.restype = ctypes.c_uint32
    plan_check.lib.spread_check.argtypes = [ctypes.c_uint32]
    assert plan_check.lib.spread_check(4096) == 0
