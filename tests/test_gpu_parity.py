"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element, on the same seeded inputs.

Bars (fp32 arithmetic on the GPU, fp64 in the oracle):
  indices and fractional positions   bit-exact
  forward, fp32 output               |y - y*| <= 1e-6 |y*| + 1e-6 max|theta|
  forward, fp16 output               |y - y*| <= 2e-3 absolute, and the tighter
                                     1e-3 |y*| + 1e-6 max|theta| + 1.2e-7 (half an fp16 ulp
                                     plus the fp32 arithmetic plus one fp16 subnormal step),
                                     which still bites for the paper's U(-1e-4,1e-4) tables
  backward (atomic order varies)     |g - g*| <= 1e-5 A, with A the sum of the absolute
                                     values of the summands of that entry (oracle run on |dL/dy|)
  backward, workspace variant        the same plus M 2^(H-54): it sums in 64-bit fixed point with
                                     each summand rounded to at most M 2^(H-62), M = max|dL/dy|,
                                     H = max(3 + ceil(log2 B), 11); the floor allows 256 such roundings.
                                     Its records carry the interpolation weights as small floats
                                     (relative precision 2^-20, exact along dimension 0 from the second
                                     voxel on, 2^-17 in the first): inside the 1e-5 A
"""
import numpy as np
import pytest
import torch

from oracle import hashgrid_oracle as orc
from paper_2201_05989_amd import HashGrid, synth

pytestmark = pytest.mark.gpu

NP = {"f32": np.float32, "f16": np.float16}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_fwd(y_gpu, y_ref, theta_absmax, io):
    y = y_gpu.astype(np.float64)
    err = np.abs(y - y_ref)
    if io == "f32":
        bound = 1e-6 * np.abs(y_ref) + 1e-6 * theta_absmax
    else:
        assert err.max() <= 2e-3
        bound = 1e-3 * np.abs(y_ref) + 1e-6 * theta_absmax + 1.2e-7
    bad = err > bound
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs off, worst err {err.max():.3e}"


def check_bwd(g_gpu, g_ref, g_abs, floor=0.0):
    err = np.abs(g_gpu.astype(np.float64) - g_ref)
    bad = err > 1e-5 * g_abs + 1e-30 + floor
    assert not bad.any(), f"{bad.sum()} of {bad.size} gradients off, worst {np.max(err / (g_abs + 1e-300)):.3e} of A"
    assert (g_gpu[g_abs == 0] == 0).all()  # entries no point touches stay exactly as they were


def same_forward(ya, yb, io):
    """Two variants of the forward kernel: the same fp32 arithmetic; with fp16 output an exact tie
    may round either way (the compiler folds the conversion into the last multiply-add of some
    instantiations), so a few outputs in a million may differ by one fp16 step."""
    if io == "f32":
        assert torch.equal(ya, yb)
        return
    ne = ya != yb
    assert int(ne.sum()) <= max(8, ya.numel() // 10000)
    a, b = ya[ne].float(), yb[ne].float()
    assert bool(((a - b).abs() <= 2.0 ** -10 * torch.maximum(a.abs(), b.abs()) + 6e-8).all())


def ws_floor(dy, B):
    H = max(3 + int(np.ceil(np.log2(max(B, 2)))), 11)  # summands carry at most 51 bits below the largest
    return float(np.abs(dy.astype(np.float64)).max()) * 2.0 ** (H - 54)


def run_case(d, L, F, T, N_min, N_max, pdt, iot, interp, x, theta, dy, do_indices=True, do_dx=True):
    cfg = orc.OracleConfig(d, L, F, T, N_min, N_max, interp)
    grid = HashGrid(d, L, F, T, N_min, N_max, pdt, iot, interp)
    lv = orc.levels(cfg)
    assert grid.n_entries == lv.total
    xd, td, gd = dev(x), dev(theta), dev(dy)
    theta_absmax = float(np.abs(theta.astype(np.float64)).max()) if theta.size else 0.0

    if do_indices:
        for l in range(L):
            idx, w = grid.debug_indices(xd, l)
            idx_ref, w_ref = orc.indices(cfg, x, l)
            np.testing.assert_array_equal(idx.cpu().numpy().view(np.uint32), idx_ref)
            np.testing.assert_array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))

    y = grid.encode_fwd(xd, td)
    check_fwd(y.cpu().numpy(), orc.encode_fwd(cfg, x, theta), theta_absmax, iot)

    g = grid.encode_bwd(xd, gd, use_workspace=False)  # hashgrid_encode_bwd: device-wide atomics
    g_ref = orc.encode_bwd(cfg, x, dy)
    g_abs = orc.encode_bwd(cfg, x, np.abs(dy.astype(np.float64)))
    check_bwd(g.cpu().numpy(), g_ref, g_abs)
    # accumulates into what is already there
    g2 = grid.encode_bwd(xd, gd, g.clone(), use_workspace=False)
    check_bwd(g2.cpu().numpy(), 2 * g_ref, 2 * g_abs)
    if grid.bwd_workspace_bytes(len(x)):             # hashgrid_encode_bwd_ws: binned, fixed-point sums
        floor = ws_floor(dy, len(x))  # the bar of the atomic pass, 1e-5 A, plus the floor of the fixed-point sums
        gw = grid.encode_bwd(xd, gd, use_workspace=True)
        check_bwd(gw.cpu().numpy(), g_ref, g_abs, floor)
        gw2 = grid.encode_bwd(xd, gd, gw.clone(), use_workspace=True)
        check_bwd(gw2.cpu().numpy(), 2 * g_ref, 2 * g_abs, 2 * floor)
        # HG_BWD_OVERWRITE: the same gradient whatever the buffer held (here NaN), untouched entries 0
        go = grid.encode_bwd(xd, gd, torch.full_like(gw, float("nan")), use_workspace=True, overwrite=True)
        check_bwd(go.cpu().numpy(), g_ref, g_abs, floor)
        # hashgrid_encode_fwd_ws: the same y, and its counts serve the backward pass
        yc = grid.encode_fwd(xd, td, count_for_bwd="always")
        same_forward(yc, y, iot)
        if grid._counted is not None:
            gc = grid.encode_bwd(xd, gd)
            assert grid._counted is None
            check_bwd(gc.cpu().numpy(), g_ref, g_abs, floor)

    if do_dx:
        dx = grid.encode_bwd_input(xd, td, gd).cpu().numpy().astype(np.float64)
        dx_ref = orc.encode_bwd_input(cfg, x, theta, dy)
        # every level contributes |dy| * (sum_m |d weight_m / d x_j| <= 2 N_l, 3 N_l with S') * max|theta|
        per_level = np.abs(dy.astype(np.float64)).reshape(len(x), L, F).sum(axis=2) @ lv.N.astype(np.float64)
        scale = per_level * 3.0 * theta_absmax
        assert (np.abs(dx - dx_ref) <= 2e-6 * scale[:, None] + 1e-30).all()
    return grid


def workload_case(name, B=None, table_scale=1e-4, **kw):
    w = synth.WORKLOADS[name]
    lv = orc.levels(orc.OracleConfig(w.d, w.L, w.F, w.T, w.N_min, w.N_max))
    x, theta, dy = synth.make_inputs(w, lv.total, B=B, table_scale=table_scale)
    return run_case(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype, 0, x, theta, dy, **kw)


def test_tiny2d_reference_config():
    workload_case("tiny2d")
    workload_case("tiny2d", table_scale=1.0)


@pytest.mark.parametrize("scale", [1e-4, 1.0])
def test_sdf3d_full_size(scale):
    workload_case("sdf3d", table_scale=scale)


@pytest.mark.parametrize("F", [1, 4, 8])
def test_headline_shape_with_other_feature_counts(F):
    # d=3 L=16 T=2^19 as in the headline configuration, F of Fig. 5; 40 001 points: 79 tiles, a ragged last one
    w = synth.WORKLOADS["sdf3d"]
    lv = orc.levels(orc.OracleConfig(w.d, w.L, F, w.T, w.N_min, w.N_max))
    rng = np.random.default_rng(100 + F)
    x = synth.points_sdf(rng, 40001, 3)
    theta = synth.make_tables(rng, lv.total, F, "f16", 1.0)
    dy = synth.make_dy(rng, len(x), w.L * F, "f16")
    grid = run_case(w.d, w.L, F, w.T, w.N_min, w.N_max, "f16", "f16", 0, x, theta, dy, do_indices=False)
    assert grid.bwd_workspace_bytes(len(x)) > 0


def test_two_rounds_of_workgroups_with_a_ragged_end():
    # from 2^19 points on the forward kernel gives every thread two points; the batch ends inside
    # a workgroup and inside a tile
    workload_case("sdf3d", B=(1 << 19) + 1531, table_scale=1.0, do_indices=False)


def test_sixteen_million_points_on_small_tables():
    # 2^24 + 3 points: 32 K tiles, 64 rounds of workgroups, every chunk shared by the maximum number
    # of accumulate workgroups, 64-bit offsets into x and y
    d, L, F, T, N_min, N_max = 2, 2, 2, 1 << 10, 4, 64
    cfg = orc.OracleConfig(d, L, F, T, N_min, N_max)
    lv = orc.levels(cfg)
    rng = np.random.default_rng(12)
    B = (1 << 24) + 3
    x = synth.points_uniform(rng, B, d)
    theta = synth.make_tables(rng, lv.total, F, "f32", 1.0)
    dy = synth.make_dy(rng, B, L * F, "f32")
    run_case(d, L, F, T, N_min, N_max, "f32", "f32", 0, x, theta, dy, do_indices=False)


def test_nerf3d_full_size():
    workload_case("nerf3d", table_scale=1.0, do_indices=False)


@pytest.mark.parametrize("B", [70001, 33, 4100])
def test_samples_in_ray_order_with_a_ragged_end(B):
    # neighbouring points share voxels and bins: the count pass folds runs of neighbouring lanes into one add and
    # the scatter pass spreads a tile's records for a bin; the batch ends inside a wave (and inside a row of 16
    # lanes), so the last wave folds runs with some of its lanes outside the batch
    w = synth.WORKLOADS["nerf3d"]
    lv = orc.levels(orc.OracleConfig(w.d, w.L, w.F, w.T, w.N_min, w.N_max))
    rng = np.random.default_rng(B)
    x = synth.points_rays(rng, B, 3)
    theta = synth.make_tables(rng, lv.total, w.F, "f16", 1.0)
    dy = synth.make_dy(rng, B, w.L * w.F, "f16")
    run_case(w.d, w.L, w.F, w.T, w.N_min, w.N_max, "f16", "f16", 0, x, theta, dy, do_indices=False)


def test_random_configurations_and_point_orders():
    # a seeded sweep over shapes, types, interpolation and the order of the points: uniform, samples along rays,
    # few distinct points in sorted order (long runs of equal bins and addresses), coordinates at 0, next to 1 and on
    # vertices, points along one row of voxels; every path of run_case on each
    for case in range(250):
        rng = np.random.default_rng(900000 + case)
        d = int(rng.choice([1, 2, 3], p=[0.15, 0.35, 0.5]))
        F = int(rng.choice([1, 2, 4, 8]))
        L = int(rng.choice([1, 2, 4, 7, 16]))
        T = int(rng.choice([1 << 10, 1 << 12, 3000, 1 << 14, 1 << 16, 100003, 1 << 19]))
        N_min = int(rng.choice([2, 4, 16]))
        N_max = N_min if L == 1 else int(N_min * rng.choice([1, 2, 8, 32, 128]))
        interp = int(rng.integers(0, 2))
        pdt, iot = str(rng.choice(["f16", "f32"])), str(rng.choice(["f16", "f32"]))
        B = int(rng.choice([1, 17, 63, 64, 65, 511, 513, 1000, 4097, 20011]))
        lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
        kind = str(rng.choice(["uniform", "rays", "dups", "edges", "line"]))
        if kind == "rays" and d == 3:
            x = synth.points_rays(rng, B, 3, samples_per_ray=int(rng.choice([16, 256, 2048])))
        elif kind == "dups":
            base = synth.points_uniform(rng, max(1, B // 50), d)
            x = np.sort(base[rng.integers(0, len(base), B)], axis=0)
        elif kind == "edges":
            x = synth.points_uniform(rng, B, d)
            m = rng.random((B, d))
            x[m < 0.2] = 0.0
            x[m > 0.8] = np.nextafter(np.float32(1.0), np.float32(0.0))
            x[(m > 0.4) & (m < 0.5)] = 0.5
        elif kind == "line":
            x = np.full((B, d), 0.3, dtype=np.float32)
            x[:, 0] = np.sort(rng.random(B).astype(np.float32)) * np.float32(0.999)
        else:
            x = synth.points_uniform(rng, B, d)
        x = np.ascontiguousarray(x, dtype=np.float32)
        theta = synth.make_tables(rng, lv.total, F, pdt, 1.0)
        dy = synth.make_dy(rng, B, L * F, iot)
        if rng.random() < 0.3:
            dy[rng.random(dy.shape) < 0.5] = 0
        try:
            run_case(d, L, F, T, N_min, N_max, pdt, iot, interp, x, theta, dy, do_indices=False, do_dx=bool(rng.random() < 0.3))
        except AssertionError as e:
            raise AssertionError(f"case {case}: d={d} L={L} F={F} T={T} N={N_min}..{N_max} interp={interp} {pdt}/{iot} "
                                 f"B={B} {kind}: {e}") from e


def test_image2d_full_size():
    workload_case("image2d", table_scale=1.0, do_indices=False)


def test_large3d_full_size_sampled_forward_and_prefix_backward():
    # 2^21 points, 777 MiB of fp16 tables: forward checked on a random sample of output rows
    # (rows are independent), backward checked in full on a 2^18-point prefix-sized draw.
    w = synth.WORKLOADS["large3d"]
    cfg = orc.OracleConfig(w.d, w.L, w.F, w.T, w.N_min, w.N_max)
    lv = orc.levels(cfg)
    x, theta, dy = synth.make_inputs(w, lv.total, table_scale=1.0)
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
    xd, td = dev(x), dev(theta)
    y = grid.encode_fwd(xd, td).cpu().numpy()
    rows = np.random.default_rng(0).choice(w.B, 1 << 16, replace=False)
    rows.sort()
    check_fwd(y[rows], orc.encode_fwd(cfg, x[rows], theta), 1.0, w.io_dtype)
    nb = 260000  # ends inside a tile of the sorted pass (here 4096 points) and inside one of its 512-point steps
    xs, dys = x[:nb], dy[:nb]
    g_ref = orc.encode_bwd(cfg, xs, dys)
    g_abs = orc.encode_bwd(cfg, xs, np.abs(dys.astype(np.float64)))
    g = grid.encode_bwd(dev(xs), dev(dys), use_workspace=False).cpu().numpy()  # atomics
    check_bwd(g, g_ref, g_abs)
    del g
    # the sorted pass: 49 K chunks, so it takes tiles of 4096 points and writes its records unstaged
    assert grid.bwd_workspace_bytes(nb) > 0
    floor = ws_floor(dys, nb)
    g = grid.encode_bwd(dev(xs), dev(dys), use_workspace=True).cpu().numpy()
    check_bwd(g, g_ref, g_abs, floor)
    del g, g_ref, g_abs
    # a batch smaller than one tile, against the atomic pass (checked above)
    few = 300
    ga = grid.encode_bwd(dev(x[:few]), dev(dy[:few]), use_workspace=False)
    gb = grid.encode_bwd(dev(x[:few]), dev(dy[:few]), use_workspace=True)
    torch.testing.assert_close(gb, ga, rtol=1e-5, atol=1e-5 * float(ga.abs().max()))


SWEEP = [
    # d, L, F, T, N_min, N_max, param, io, interp, B
    (1, 5, 1, 64, 2, 300, "f32", "f32", 0, 1000),
    (1, 3, 8, 1 << 8, 4, 64, "f16", "f32", 1, 777),
    (2, 6, 1, 1 << 9, 4, 100, "f16", "f16", 0, 2049),
    (2, 6, 4, 1 << 9, 4, 100, "f32", "f16", 1, 513),
    (2, 4, 8, 1000, 3, 50, "f32", "f32", 0, 300),        # T not a power of two
    (3, 8, 1, 1 << 12, 4, 128, "f32", "f32", 0, 4097),
    (3, 8, 2, 1 << 12, 4, 128, "f16", "f16", 1, 4097),
    (3, 8, 4, 1 << 12, 4, 128, "f16", "f32", 0, 1025),
    (3, 8, 8, 1 << 12, 4, 128, "f32", "f16", 0, 255),
    (3, 5, 2, 4099, 2, 40, "f16", "f16", 0, 1500),       # prime T
    (3, 32, 2, 1 << 14, 16, 2048, "f16", "f16", 0, 3000),  # L = 32
    (3, 1, 2, 1 << 19, 16, 16, "f32", "f32", 0, 100),     # single level
    (3, 16, 2, 1 << 19, 16, 2048, "f32", "f32", 0, 10000),
    (3, 16, 2, 1 << 19, 16, 2048, "f16", "f32", 1, 10000),
    (2, 16, 2, 1 << 15, 16, 2048, "f16", "f16", 0, 1),    # one point
    (3, 4, 2, 1, 2, 16, "f32", "f32", 0, 200),            # T = 1: every corner collides
]


@pytest.mark.parametrize("d,L,F,T,N_min,N_max,pdt,iot,interp,B", SWEEP)
def test_sweep_of_shapes_and_dtypes(d, L, F, T, N_min, N_max, pdt, iot, interp, B):
    rng = np.random.default_rng(1000 + B)
    lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
    x = synth.points_uniform(rng, B, d)
    theta = synth.make_tables(rng, lv.total, F, pdt, 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    run_case(d, L, F, T, N_min, N_max, pdt, iot, interp, x, theta, dy)


def _random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.integers(1, 4))
    F = int(rng.choice([1, 2, 4, 8]))
    L = int(rng.integers(1, 13))
    T = int(rng.choice([1 << int(rng.integers(0, 18)), int(rng.integers(1, 100000))], p=[0.8, 0.2]))
    N_min = int(rng.integers(1, 40))
    N_max = int(N_min * rng.choice([1, 2, 7, 100, 3000]) + rng.integers(0, 5))
    pdt, iot = (str(rng.choice(["f16", "f32"])) for _ in range(2))
    interp = int(rng.integers(0, 2))
    B = int(rng.choice([1, 63, 512, 513, int(rng.integers(2, 3000))]))
    return d, L, F, T, N_min, N_max, pdt, iot, interp, B


@pytest.mark.parametrize("seed", range(32))
def test_random_configurations(seed):
    # seeded draws over every parameter of the configuration, including tables smaller than a chunk,
    # resolutions beyond 4096, single levels and single points: every entry point against the oracle
    d, L, F, T, N_min, N_max, pdt, iot, interp, B = _random_case(seed)
    lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
    rng = np.random.default_rng(5000 + seed)
    x = synth.points_uniform(rng, B, d)
    theta = synth.make_tables(rng, lv.total, F, pdt, 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    run_case(d, L, F, T, N_min, N_max, pdt, iot, interp, x, theta, dy)


@pytest.mark.parametrize("d,L,F,T,N_min,N_max,pdt,iot,interp,B", [
    (3, 16, 2, 1000003, 16, 2048, "f16", "f16", 0, 40001),    # the headline shape with T not a power of two
    (3, 8, 2, 524287, 16, 512, "f16", "f32", 1, 20000),       # a prime T (2^19 - 1), smoothstep
    (2, 10, 4, 3 * (1 << 18), 16, 8192, "f32", "f16", 0, 33333),  # 3 * 2^18: resolutions beyond one chunk
    (3, 6, 8, 100003, 8, 300, "f16", "f32", 0, 9001),         # 40-byte records, eight per point and level: unstaged
    (1, 12, 2, 1 << 16, 16, 1 << 20, "f16", "f16", 0, 50000),  # one dimension: 1:1 levels longer than a chunk
    (1, 8, 1, 5000, 16, 1 << 18, "f32", "f32", 1, 12345),
])
def test_sorted_backward_with_a_record_per_corner(d, L, F, T, N_min, N_max, pdt, iot, interp, B):
    # Eq. 4's mod T with a T that is not a power of two, and d = 1: the two corners of a pair are not
    # neighbours in memory, so the sorted pass gives every corner its own record; batches of many tiles
    # with a ragged last one, every entry point against the oracle
    cfg = orc.OracleConfig(d, L, F, T, N_min, N_max, interp)
    lv = orc.levels(cfg)
    rng = np.random.default_rng(77 + B)
    x = synth.points_uniform(rng, B, d)
    x[:20] = 0.0
    x[20:40] = 1 - 2.0 ** -24
    theta = synth.make_tables(rng, lv.total, F, pdt, 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    grid = run_case(d, L, F, T, N_min, N_max, pdt, iot, interp, x, theta, dy, do_indices=False)
    assert grid.bwd_workspace_bytes(B) > 0 and grid.bwd_ws_pays(B)


@pytest.mark.parametrize("seed", range(24))
def test_random_larger_configurations(seed):
    # seeded draws with batches of many tiles (5 K to 150 K points, uniform or near a surface), tables
    # of up to 2^21 entries per level and up to 16 levels: the sorted backward pass with several
    # slices per chunk, level parts and ragged last tiles, against the oracle
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.integers(2, 4))
    F = int(rng.choice([1, 2, 4, 8]))
    L = int(rng.choice([2, 4, 8, 16]))
    T = 1 << int(rng.integers(10, 22))
    N_min = int(rng.integers(2, 40))
    N_max = int(N_min * rng.choice([2, 16, 128, 1000]) + rng.integers(0, 5))
    pdt, iot = (str(rng.choice(["f16", "f32"])) for _ in range(2))
    interp = int(rng.integers(0, 2))
    B = int(rng.integers(5000, 150000))
    lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
    kind = str(rng.choice(["uniform", "sdf"])) if d == 3 else "uniform"
    x = synth.points_uniform(rng, B, d) if kind == "uniform" else synth.points_sdf(rng, B)
    theta = synth.make_tables(rng, lv.total, F, pdt, 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    run_case(d, L, F, T, N_min, N_max, pdt, iot, interp, x, theta, dy, do_indices=False)


def test_edge_positions_and_grid_vertices():
    # exact 0, the largest fp32 below 1, grid vertices of every level and their fp32 neighbours
    d, L, F, T, N_min, N_max = 3, 8, 2, 1 << 12, 4, 512
    lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max))
    rng = np.random.default_rng(3)
    pts = [np.zeros((1, 3)), np.full((1, 3), 1 - 2.0 ** -24)]
    for N in lv.N:
        k = rng.integers(0, int(N), (64, 3))
        v = (k / float(N)).astype(np.float32)
        pts += [v, np.nextafter(v, np.float32(0)), np.nextafter(v, np.float32(1))]
    x = np.clip(np.concatenate(pts).astype(np.float32), 0, np.float32(1 - 2.0 ** -24))
    dy = synth.make_dy(rng, len(x), L * F, "f32")
    for interp in (0, 1):
        lvi = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
        th = synth.make_tables(rng, lvi.total, F, "f32", 1.0)
        run_case(d, L, F, T, N_min, N_max, "f32", "f32", interp, x, th, dy, do_dx=False)


@pytest.mark.parametrize("d", [2, 3])
@pytest.mark.parametrize("iot", ["f16", "f32"])
def test_workspace_backward_when_pairs_straddle_two_chunks(d, iot):
    # resolutions of 4096 and more on hashed levels: where the voxel coordinate along dimension 0
    # ends in twelve one bits, its two corners hash into different 4096-entry chunks.  Half of the
    # points sit in such voxels on every level, the rest are uniform.
    L, F, T, N_min, N_max = 3, 2, 1 << 16, 8192, 32768
    cfg = orc.OracleConfig(d, L, F, T, N_min, N_max)
    lv = orc.levels(cfg)
    assert not lv.dense.any()
    rng = np.random.default_rng(77)
    B = 6000
    x = synth.points_uniform(rng, B, d)
    k = rng.integers(0, 2, B // 2)
    x[: B // 2, 0] = ((4095.75 + 4096.0 * k) / 8192.0).astype(np.float32)  # 4095 mod 4096 at every level
    for l in range(L):
        c0 = np.floor(x[: B // 2, 0].astype(np.float32) * np.float32(lv.N[l])).astype(np.int64)
        assert ((c0 & 4095) == 4095).all()
    theta = synth.make_tables(rng, lv.total, F, "f16", 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    grid = run_case(d, L, F, T, N_min, N_max, "f16", iot, 0, x, theta, dy, do_dx=False)
    assert grid.bwd_workspace_bytes(B) > 0


@pytest.mark.parametrize("d,F,iot,interp,B", [(2, 1, "f32", 1, 9000), (3, 2, "f16", 0, 4096 + 513)])
def test_workspace_backward_with_very_many_chunks(d, F, iot, interp, B):
    # more than 16 K chunks in all: the sorted pass takes tiles of 4096 points and writes its records
    # unstaged.  Five hashed levels of 2^24 entries, resolutions of 4096 and more (pairs that straddle
    # two chunks occur too); the batch ends inside a tile and inside one of its 512-point steps.
    L, T, N_min, N_max = 5, 1 << 24, 8192, 65536
    lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
    assert not lv.dense.any()
    rng = np.random.default_rng(78)
    x = synth.points_uniform(rng, B, d)
    x[: B // 4, 0] = ((4095.75 + 4096.0 * rng.integers(0, 2, B // 4)) / 8192.0).astype(np.float32)
    theta = synth.make_tables(rng, lv.total, F, "f16", 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    grid = run_case(d, L, F, T, N_min, N_max, "f16", iot, interp, x, theta, dy, do_dx=False, do_indices=False)
    assert grid.bwd_workspace_bytes(B) > 0


@pytest.mark.parametrize("F,pdt,iot,shift", [(2, "f16", "f16", None), (1, "f32", "f16", None), (4, "f16", "f32", None),
                                             (8, "f32", "f32", 4)])
def test_buffers_aligned_to_one_entry_only(F, pdt, iot, shift):
    # every array starts one table entry (one level's outputs) past a 256-byte boundary: allowed by
    # the interface, but not the 16-byte alignment the vector paths of the kernels want.  Last row:
    # 32-byte entries and output rows that start 16 bytes past a 32-byte boundary (the widest
    # alignment the entry points may assume is 16 bytes)
    d, L, T, N_min, N_max, B = 3, 8, 1 << 12, 4, 128, 3000
    cfg = orc.OracleConfig(d, L, F, T, N_min, N_max)
    lv = orc.levels(cfg)
    rng = np.random.default_rng(31)
    x = synth.points_uniform(rng, B, d)
    theta = synth.make_tables(rng, lv.total, F, pdt, 1.0)
    dy = synth.make_dy(rng, B, L * F, iot)
    grid = HashGrid(d, L, F, T, N_min, N_max, pdt, iot)

    def shifted(a, fill=None):
        k = F if shift is None else shift
        t = torch.empty(a.size + k, dtype=torch.from_numpy(a[:0]).dtype, device="cuda")
        v = t[k:].view(a.shape)
        assert v.data_ptr() % 16 != 0 or F * a.itemsize >= 16
        assert shift is None or v.data_ptr() % 32 == 16
        v.copy_(dev(a)) if fill is None else v.fill_(fill)
        return v

    td, gd = shifted(theta), shifted(dy)
    xd = dev(x)
    y = shifted(np.empty((B, L * F), NP[iot]), fill=0.0)
    grid.encode_fwd(xd, td, y)
    check_fwd(y.cpu().numpy(), orc.encode_fwd(cfg, x, theta), 1.0, iot)
    g_ref = orc.encode_bwd(cfg, x, dy)
    g_abs = orc.encode_bwd(cfg, x, np.abs(dy.astype(np.float64)))
    floor = ws_floor(dy, B)
    for use_ws, ow in ((False, False), (True, False), (True, True)):
        g = shifted(np.empty((lv.total, F), np.float32), fill=0.0)
        grid.encode_bwd(xd, gd, g, use_workspace=use_ws, overwrite=ow)
        check_bwd(g.cpu().numpy(), g_ref, g_abs, floor if use_ws else 0.0)
    y2 = shifted(np.empty((B, L * F), NP[iot]), fill=0.0)
    grid.encode_fwd(xd, td, y2, count_for_bwd="always")
    same_forward(y2, y, iot)
    g = shifted(np.empty((lv.total, F), np.float32), fill=0.0)
    grid.encode_bwd(xd, gd, g)
    check_bwd(g.cpu().numpy(), g_ref, g_abs, floor)
    dx = grid.encode_bwd_input(xd, td, gd).cpu().numpy().astype(np.float64)
    dx_ref = orc.encode_bwd_input(cfg, x, theta, dy)
    scale = np.abs(dy.astype(np.float64)).reshape(B, L, F).sum(axis=2) @ lv.N.astype(np.float64) * 3.0
    assert (np.abs(dx - dx_ref) <= 2e-6 * scale[:, None] + 1e-30).all()


def test_empty_batch_is_a_no_op():
    grid = HashGrid(3, 16, 2, 1 << 19, 16, 2048)
    x = torch.empty((0, 3), dtype=torch.float32, device="cuda")
    theta = torch.zeros((grid.n_entries, 2), dtype=torch.float16, device="cuda")
    y = grid.encode_fwd(x, theta)
    assert y.shape == (0, 32)
    g = grid.encode_bwd(x, torch.empty((0, 32), dtype=torch.float16, device="cuda"))
    assert float(g.abs().max()) == 0.0


def test_precondition_check_counts_coordinates_outside_the_unit_interval():
    grid = HashGrid(3, 4, 2, 1 << 12, 4, 64)
    rng = np.random.default_rng(2)
    x = synth.points_uniform(rng, 100003, 3)
    assert grid.debug_count_outside(dev(x)) == 0
    x[5, 0], x[77, 2], x[4000, 1], x[99999, 0], x[100002, 2] = 1.0, -1e-9, np.nan, np.inf, 7.0
    x[10, 1] = np.float32(1 - 2.0 ** -24)   # the largest float below 1 is inside
    x[11, 1] = -0.0                          # and so is a negative zero
    assert grid.debug_count_outside(dev(x)) == 5


def test_out_of_range_positions_stay_in_bounds():
    # a violated precondition must not fault: values are unspecified, memory safety is not
    grid = HashGrid(3, 16, 2, 1 << 19, 16, 2048, "f32", "f32")
    bad = np.array([[1.0, 0.5, 0.5], [-0.25, 0.5, 0.5], [0.5, 2.0, 1e9], [np.nan, np.inf, -np.inf],
                    [0.5, 0.5, 0.5]], np.float32)
    x = dev(bad)
    theta = torch.ones((grid.n_entries, 2), dtype=torch.float32, device="cuda")
    y = grid.encode_fwd(x, theta)
    g = grid.encode_bwd(x, torch.ones((5, 32), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    np.testing.assert_allclose(y[4].cpu().numpy(), 1.0, rtol=1e-6)
    assert g.shape == (grid.n_entries, 2)


def test_non_default_stream():
    w = synth.WORKLOADS["tiny2d"]
    cfg = orc.OracleConfig(w.d, w.L, w.F, w.T, w.N_min, w.N_max)
    lv = orc.levels(cfg)
    x, theta, dy = synth.make_inputs(w, lv.total, table_scale=1.0)
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, "f32", "f32")
    xd, td = dev(x), dev(theta)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        y = grid.encode_fwd(xd, td)
    s.synchronize()
    check_fwd(y.cpu().numpy(), orc.encode_fwd(cfg, x, theta), 1.0, "f32")


def test_two_streams_share_a_handle_with_a_workspace_each():
    # the handle is read-only; calls that overlap in time need their own scratch buffers
    w = synth.WORKLOADS["sdf3d"]
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
    B = 40000
    x, theta, dy = synth.make_inputs(w, grid.n_entries, B=2 * B, table_scale=1.0)
    xs, dys = [dev(x[:B]), dev(x[B:])], [dev(dy[:B]), dev(dy[B:])]
    ref = [grid.encode_bwd(xs[i], dys[i], use_workspace=True) for i in range(2)]
    need = grid.bwd_workspace_bytes(B)
    spaces = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(2)]
    grads = [torch.zeros_like(ref[0]) for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    for _ in range(3):  # several rounds in flight on both streams at once
        for i in range(2):
            grid.encode_bwd(xs[i], dys[i], grads[i], stream=streams[i], workspace=spaces[i], use_workspace=True,
                            overwrite=True)
    torch.cuda.synchronize()
    hashed_from = [i for i in grid.levels() if not i.is_dense][0].entry_offset
    for i in range(2):
        assert torch.equal(grads[i][hashed_from:], ref[i][hashed_from:])
        torch.testing.assert_close(grads[i][:hashed_from], ref[i][:hashed_from], rtol=1e-4,
                                   atol=1e-4 * float(ref[i].abs().max()))


def test_workspace_backward_is_reproducible_and_keeps_untouched_entries():
    w = synth.WORKLOADS["sdf3d"]
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
    x, _, dy = synth.make_inputs(w, grid.n_entries, B=50000)
    xd, gd = dev(x), dev(dy)
    assert grid.bwd_workspace_bytes(len(x)) > 0
    g1 = grid.encode_bwd(xd, gd, use_workspace=True)
    g2 = grid.encode_bwd(xd, gd, use_workspace=True)
    hashed = [i for i in grid.levels() if not i.is_dense]
    lo = hashed[0].entry_offset
    # hashed levels: one owner per chunk, exact fixed-point sums: bit-for-bit equal run to run
    assert torch.equal(g1[lo:], g2[lo:])
    # entries no point reaches keep their previous bits (here a sentinel)
    sentinel = torch.full((grid.n_entries, 2), 7.25, dtype=torch.float32, device="cuda")
    g3 = grid.encode_bwd(xd, gd, sentinel.clone(), use_workspace=True)
    untouched = (g1 == 0).all(dim=1)
    assert untouched.any() and bool((g3[untouched] == 7.25).all())


def test_counting_forward_gives_the_counts_of_the_count_pass():
    # bit-for-bit the same gradient on hashed levels (exact sums), with and without the counting pass
    for name, B in (("sdf3d", 70001), ("tiny2d", 4096), ("image2d", 30000)):
        w = synth.WORKLOADS[name]
        grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
        x, theta, dy = synth.make_inputs(w, grid.n_entries, B=B, table_scale=1.0)
        xd, td, gd = dev(x), dev(theta), dev(dy)
        y0 = grid.encode_fwd(xd, td)
        g0 = grid.encode_bwd(xd, gd, use_workspace=True)
        y1 = grid.encode_fwd(xd, td, count_for_bwd="always")
        counted = grid._counted is not None
        g1 = grid.encode_bwd(xd, gd, use_workspace=True)
        same_forward(y0, y1, w.io_dtype)
        hashed = [i for i in grid.levels() if not i.is_dense]
        lo = hashed[0].entry_offset
        assert torch.equal(g0[lo:], g1[lo:])
        torch.testing.assert_close(g0[:lo], g1[:lo], rtol=1e-4, atol=1e-4 * float(g0.abs().max()))
        assert counted
        # the counts are consumed: a second backward counts for itself and agrees
        g2 = grid.encode_bwd(xd, gd, use_workspace=True)
        assert torch.equal(g0[lo:], g2[lo:])
        # points changed in place after the forward pass: the binding drops the counts (they belong to
        # the old points) and the backward pass counts for itself
        grid.encode_fwd(xd, td, count_for_bwd="always")
        xd2 = xd.clone()
        xd.copy_(xd.flip(0))
        g3 = grid.encode_bwd(xd, gd, use_workspace=True)
        g4 = grid.encode_bwd(xd.clone(), gd, use_workspace=True)
        assert torch.equal(g3[lo:], g4[lo:])
        xd.copy_(xd2)


def test_step_replays_from_a_hip_graph():
    # the library launches kernels only (no allocation, no memset, no synchronisation), so a step can
    # be captured once and replayed; replays interleaved with eager work must reproduce the eager result
    w = synth.WORKLOADS["sdf3d"]
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
    B = 40000
    x, theta, dy = synth.make_inputs(w, grid.n_entries, B=B, table_scale=1.0)
    xd, td, gd = dev(x), dev(theta), dev(dy)
    y_ref = grid.encode_fwd(xd, td, count_for_bwd="always")       # also allocates the scratch buffer
    g_ref = grid.encode_bwd(xd, gd)
    y = torch.zeros_like(y_ref)
    grad = torch.zeros_like(g_ref)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            grad.fill_(0.0)                                       # a fill kernel, not a memset node
            grid.encode_fwd(xd, td, y, count_for_bwd="always")
            grid.encode_bwd(xd, gd, grad)
    torch.cuda.current_stream().wait_stream(side)
    hashed_from = [i for i in grid.levels() if not i.is_dense][0].entry_offset
    for k in range(4):
        y.zero_()
        grad.fill_(float(k))                                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        same_forward(y, y_ref, w.io_dtype)
        assert torch.equal(grad[hashed_from:], g_ref[hashed_from:])
        torch.testing.assert_close(grad[:hashed_from], g_ref[:hashed_from], rtol=1e-4,
                                   atol=1e-4 * float(g_ref.abs().max()))


def test_binding_picks_the_backward_pass_by_batch_size():
    grid = HashGrid(3, 16, 2, 1 << 19, 16, 2048)
    assert not grid.bwd_ws_pays(1024) and grid.bwd_ws_pays(1 << 16)
    assert not HashGrid(3, 2, 2, 1 << 25, 16, 2048).bwd_ws_pays(1 << 20)  # not served at all (too many chunks per level)
    for B in (1000, 1 << 16):
        x = torch.rand((B, 3), device="cuda") * 0.99
        dy = torch.randn((B, 32), device="cuda").half()
        ga = grid.encode_bwd(x, dy)                        # the binding's choice
        gb = grid.encode_bwd(x, dy, use_workspace=False)   # atomics
        torch.testing.assert_close(ga, gb, rtol=1e-4, atol=1e-4 * float(gb.abs().max()))
        assert bool(grid._ws) == (B == 1 << 16)            # the scratch buffer appears only when the sort is used


def test_workspace_backward_argument_checks():
    grid = HashGrid(3, 16, 2, 1 << 19, 16, 2048)
    B = 1000
    need = grid.bwd_workspace_bytes(B)
    assert need > B * 16 * 4 * 12  # 12-byte records for fp16 dL/dy
    x = torch.rand((B, 3), device="cuda") * 0.99
    dy = torch.ones((B, 32), dtype=torch.float16, device="cuda")
    g = torch.zeros((grid.n_entries, 2), dtype=torch.float32, device="cuda")
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    lib = grid._lib
    st = lib.hashgrid_encode_bwd_ws(grid._h, B, x.data_ptr(), dy.data_ptr(), g.data_ptr(), small.data_ptr(),
                                    small.numel(), 0, None)
    assert st == 1  # too small
    st = lib.hashgrid_encode_bwd_ws(grid._h, B, x.data_ptr(), dy.data_ptr(), g.data_ptr(), None, need, 0, None)
    assert st == 1
    big = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert lib.hashgrid_encode_bwd_ws(grid._h, B, x.data_ptr(), dy.data_ptr(), g.data_ptr(), big.data_ptr(), need,
                                      8, None) == 1  # unknown flag
    # configurations the binned path does not serve report 0 bytes and HG_ERR_UNSUPPORTED
    g4 = HashGrid(3, 2, 4, 1 << 25, 16, 2048)  # more than 4096 chunks per level
    assert g4.bwd_workspace_bytes(B) == 0
    assert lib.hashgrid_encode_bwd_ws(g4._h, B, x.data_ptr(), dy.data_ptr(), g.data_ptr(), small.data_ptr(),
                                      small.numel(), 0, None) == 2
    assert lib.hashgrid_encode_fwd_ws(g4._h, B, x.data_ptr(), x.data_ptr(), x.data_ptr(), small.data_ptr(),
                                      small.numel(), None) == 2
    # a table size that is not a power of two: the sorted pass serves it with a record per corner
    g5 = HashGrid(3, 16, 4, 1000003, 16, 2048)
    assert g5.bwd_workspace_bytes(B) > B * 16 * 8 * 16


def test_workspace_backward_with_non_finite_upstream_gradient():
    # inf / NaN in dL/dy must reach exactly the entries the oracle says they reach
    d, L, F, T, N_min, N_max = 3, 6, 2, 1 << 14, 8, 256
    cfg = orc.OracleConfig(d, L, F, T, N_min, N_max)
    grid = HashGrid(d, L, F, T, N_min, N_max, "f16", "f32")
    rng = np.random.default_rng(21)
    x = synth.points_uniform(rng, 3000, d)
    dy = synth.make_dy(rng, 3000, L * F, "f32")
    dy[17, 3] = np.inf
    dy[99, 8] = np.nan
    with np.errstate(invalid="ignore"):
        ref = orc.encode_bwd(cfg, x, dy)
    for use_ws, overwrite in ((False, False), (True, False), (True, True)):
        old = torch.full((grid.n_entries, F), 7.0, device="cuda") if overwrite else None
        g = grid.encode_bwd(dev(x), dev(dy), old, use_workspace=use_ws, overwrite=overwrite).cpu().numpy()
        assert (np.isfinite(g) == np.isfinite(ref)).all()
        assert (np.isnan(g) == np.isnan(ref)).all()
        fin = np.isfinite(ref)
        np.testing.assert_allclose(g[fin], ref[fin], rtol=1e-4, atol=1e-5)


def test_overwriting_backward():
    # HG_BWD_OVERWRITE at the headline shape (several slices per chunk on the coarse levels), with
    # the counts of the forward pass, on a buffer full of other values: equal to the adding call on
    # zeros where one workgroup owns a chunk, and within rounding of it where several add up;
    # a batch of zeros clears the buffer; the atomic pass behind the same option of the binding.
    w = synth.WORKLOADS["sdf3d"]
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, w.param_dtype, w.io_dtype)
    x, theta, dy = synth.make_inputs(w, grid.n_entries, B=50000, table_scale=1.0)
    xd, td, gd = dev(x), dev(theta), dev(dy)
    g_add = grid.encode_bwd(xd, gd, use_workspace=True)
    junk = torch.randn((grid.n_entries, w.F), device="cuda")
    grid.encode_fwd(xd, td, count_for_bwd="always")
    g_ow = grid.encode_bwd(xd, gd, junk.clone(), overwrite=True)
    hashed_from = [i for i in grid.levels() if not i.is_dense][0].entry_offset
    assert torch.equal(g_ow[hashed_from:], g_add[hashed_from:])
    torch.testing.assert_close(g_ow[:hashed_from], g_add[:hashed_from], rtol=1e-4,
                               atol=1e-4 * float(g_add.abs().max()))
    g0 = grid.encode_bwd(xd, torch.zeros_like(gd), junk.clone(), use_workspace=True, overwrite=True)
    assert not g0.any()
    ga = grid.encode_bwd(xd[:1000], gd[:1000], junk.clone(), use_workspace=False, overwrite=True)
    gb = grid.encode_bwd(xd[:1000], gd[:1000], use_workspace=False)
    torch.testing.assert_close(ga, gb, rtol=1e-4, atol=1e-4 * float(gb.abs().max()))
