"""Pins for the CPU oracle: everything here checks the oracle against facts the
paper or the mathematics fix, never against itself and never against the GPU
library.  Citations are to the paper's sections, equations and figures."""
import os
from decimal import Decimal, getcontext

import numpy as np
import pytest
import scipy.ndimage

from oracle import hashgrid_oracle as orc
from oracle.hashgrid_oracle import OracleConfig

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if line:
            out.append(line.split())
    return out


# ----------------------------------------------------------------------------- level table (Eq. 2-3)

TABLE1_CFGS = [(2, 4, 1 << 10, 4, 32), (2, 16, 1 << 22, 16, 32768), (3, 16, 1 << 19, 16, 2048),
               (3, 16, 1 << 24, 16, 524288), (3, 16, 1 << 19, 16, 512), (3, 16, 1 << 14, 16, 4096),
               (2, 16, 1 << 22, 16, 11733), (3, 8, 1 << 19, 16, 1000), (3, 32, 1 << 19, 16, 2048)]


def _levels_decimal(L, N_min, N_max):
    """Eq. 2-3 in 60-digit decimal arithmetic: floor(N_min * (N_max/N_min)^(l/(L-1)))."""
    getcontext().prec = 60
    out = []
    for l in range(L):
        if L == 1:
            out.append(N_min)
            continue
        ln_b = (Decimal(N_max).ln() - Decimal(N_min).ln()) / Decimal(L - 1)
        s = Decimal(N_min) * (ln_b * l).exp()
        near = s.to_integral_value()
        # levels whose real value is an integer (b^l rational power landing on one)
        if abs(s - near) < Decimal(10) ** -40:
            out.append(int(near))
        else:
            out.append(int(s.to_integral_value(rounding="ROUND_FLOOR")))
    return out


@pytest.mark.parametrize("d,L,T,N_min,N_max", TABLE1_CFGS)
def test_levels_match_high_precision_eq2(d, L, T, N_min, N_max):
    lv = orc.levels(OracleConfig(d, L, 2, T, N_min, N_max))
    assert list(map(int, lv.N)) == _levels_decimal(L, N_min, N_max)
    assert lv.N[0] == N_min and lv.N[-1] == N_max  # progression spans [N_min, N_max] (Section 3)


def test_levels_growth_factor_two_is_exact_doubling():
    # b = 2 when N_max/N_min = 2^(L-1): N_l = N_min 2^l exactly (Eq. 2)
    lv = orc.levels(OracleConfig(2, 4, 2, 1 << 10, 4, 32))
    assert list(lv.N) == [4, 8, 16, 32]
    lv = orc.levels(OracleConfig(3, 16, 2, 1 << 24, 16, 524288))
    assert list(lv.N) == [16 << l for l in range(16)]


def test_growth_factor_range_of_table1():
    # Section 3: b in [1.26, 2] for N_max from 512 to 524288 with N_min=16, L=16
    for N_max, b_expect in ((512, 1.26), (524288, 2.0)):
        lv = orc.levels(OracleConfig(3, 16, 2, 1 << 19, 16, N_max))
        b = (float(lv.N[-1]) / float(lv.N[0])) ** (1.0 / 15.0)
        assert abs(b - b_expect) < 5e-3


def test_single_level_is_N_min():
    lv = orc.levels(OracleConfig(3, 1, 2, 1 << 19, 16, 2048))
    assert list(lv.N) == [16]


@pytest.mark.parametrize("d,L,T,N_min,N_max", TABLE1_CFGS)
def test_dense_criterion_and_sizes(d, L, T, N_min, N_max):
    # Section 3: 1:1 when (N_l+1)^d <= T, else a table of T entries; total <= T*L (bound T*L*F on parameters)
    lv = orc.levels(OracleConfig(d, L, 2, T, N_min, N_max))
    off = 0
    for l in range(L):
        verts = (int(lv.N[l]) + 1) ** d
        assert bool(lv.dense[l]) == (verts <= T)
        assert int(lv.size[l]) == (verts if verts <= T else T)
        assert int(lv.offset[l]) == off
        off += int(lv.size[l])
    assert lv.total == off <= T * L


def test_printed_parameter_counts():
    for d, L, F, lt, N_min, N_max, mlp, printed, unit in _rows("param_counts.txt"):
        lv = orc.levels(OracleConfig(int(d), int(L), int(F), 1 << int(lt), int(N_min), int(N_max)))
        params = lv.total * int(F) + int(mlp)
        if unit == "M":
            assert round(params / 1e6, 1) == float(printed), (params, printed)
        else:
            assert round(params / 1e3) == float(printed), (params, printed)


def test_printed_count_rejects_other_size_rule():
    # a planted mistake: sizing dense levels as N_l^d instead of (N_l+1)^d misses Fig. 7's 12.2M
    lv = orc.levels(OracleConfig(3, 16, 2, 1 << 19, 16, 2048))
    wrong = sum(min(1 << 19, int(n) ** 3) for n in lv.N) * 2 + 6208
    assert round(wrong / 1e6, 1) != 12.2


# ----------------------------------------------------------------------------- hash (Eq. 4)

def test_hash_hand_values():
    for d, v0, v1, v2, lt, expect in _rows("hash_values.txt"):
        d = int(d)
        v = [int(v0), int(v1), int(v2)][:d]
        assert orc.index(d, 0, 1 << int(lt), False, v) == int(expect)


def test_hash_matches_bigint_eq4_random_vertices_and_non_pow2_T():
    rng = np.random.default_rng(5)
    primes = (1, 2654435761, 805459861)
    for T in (1 << 14, 1 << 19, 1 << 24, 1000003, 12345):
        for d in (1, 2, 3):
            for v in rng.integers(0, 1 << 20, size=(50, d)):
                h = 0
                for i in range(d):
                    h ^= (int(v[i]) * primes[i]) & 0xFFFFFFFF  # 32-bit wrap-around
                assert orc.index(d, 0, T, False, v) == h % T


def test_hash_first_dimension_is_identity_on_low_bits():
    # pi_1 = 1 (Eq. 4): for v_1 = v_2 = 0 the hash of (k,0,0) is k mod T
    for k in (0, 1, 2, 1023, 1024, 5000):
        assert orc.index(3, 0, 1 << 10, False, [k, 0, 0]) == k % 1024


# ----------------------------------------------------------------------------- dense map is 1:1 (Section 3)

@pytest.mark.parametrize("d,N", [(1, 100), (2, 4), (2, 337), (3, 16), (3, 58)])
def test_dense_map_is_bijection(d, N):
    T = (N + 1) ** d
    grids = np.meshgrid(*[np.arange(N + 1, dtype=np.uint32)] * d, indexing="ij")
    verts = np.stack([g.ravel() for g in grids], axis=1)
    idx = np.array([orc.index(d, N + 1, T, True, v) for v in verts])
    assert sorted(idx.tolist()) == list(range(T))
    # dimension 0 is the fastest-varying one (same role as pi_1 = 1 in Eq. 4)
    assert orc.index(d, N + 1, T, True, [1] + [0] * (d - 1)) == 1


def test_indices_of_dense_levels_cover_only_valid_entries():
    cfg = OracleConfig(3, 16, 2, 1 << 19, 16, 2048)
    lv = orc.levels(cfg)
    x = np.random.default_rng(0).random((2000, 3)).astype(np.float32)
    x[0] = [0.0, 0.0, 0.0]
    x[1] = [np.nextafter(np.float32(1), np.float32(0))] * 3
    for l in range(cfg.L):
        idx, w = orc.indices(cfg, x, l)
        assert idx.max() < lv.size[l]
        assert (w >= 0).all() and (w < 1).all()


# ----------------------------------------------------------------------------- interpolation (Section 3)

def _rand_cfg_inputs(cfg, B, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    lv = orc.levels(cfg)
    x = rng.random((B, cfg.d)).astype(np.float32)
    theta = rng.uniform(-scale, scale, (lv.total, cfg.F))
    return lv, x, theta


@pytest.mark.parametrize("interp", [0, 1])
@pytest.mark.parametrize("d", [1, 2, 3])
def test_constant_table_gives_constant_output(d, interp):
    # weights of d-linear interpolation are a partition of unity
    cfg = OracleConfig(d, 6, 3, 1 << 12, 4, 200, interp)
    lv, x, _ = _rand_cfg_inputs(cfg, 500, 1)
    theta = np.full((lv.total, cfg.F), 0.75)
    y = orc.encode_fwd(cfg, x, theta)
    np.testing.assert_allclose(y, 0.75, rtol=0, atol=1e-15)


@pytest.mark.parametrize("d", [2, 3])
def test_vertex_exactness_dense_and_hashed(d):
    # at a grid vertex x = k / N_l (N_l a power of two, so exact in fp32) the level's
    # output is the table entry of that vertex: dense map on coarse levels, Eq. 4 on fine ones
    cfg = OracleConfig(d, 4, 2, 1 << 10, 4, 32)
    lv = orc.levels(cfg)
    rng = np.random.default_rng(2)
    theta = rng.uniform(-1, 1, (lv.total, cfg.F))
    primes = (1, 2654435761, 805459861)
    for l in range(cfg.L):
        N = int(lv.N[l])
        k = rng.integers(0, N, size=(40, d))
        x = (k / N).astype(np.float32)
        y = orc.encode_fwd(cfg, x, theta)
        for b in range(len(k)):
            if lv.dense[l]:
                e = sum(int(k[b, i]) * (N + 1) ** i for i in range(d))
            else:
                h = 0
                for i in range(d):
                    h ^= (int(k[b, i]) * primes[i]) & 0xFFFFFFFF
                e = h % cfg.T
            np.testing.assert_array_equal(y[b, l * 2:(l + 1) * 2], theta[int(lv.offset[l]) + e])
    assert not lv.dense[-1] and lv.dense[0]


@pytest.mark.parametrize("d,N", [(2, 37), (3, 16), (3, 21)])
def test_single_dense_level_equals_library_linear_interpolation(d, N):
    # L = 1 on a 1:1 level is textbook d-linear interpolation on an (N+1)^d lattice
    # sampled at x*N: scipy.ndimage.map_coordinates(order=1) is the third opinion.
    cfg = OracleConfig(d, 1, 1, (N + 1) ** d, N, N)
    lv, x, theta = _rand_cfg_inputs(cfg, 3000, 3)
    assert lv.dense[0] and lv.total == (N + 1) ** d
    y = orc.encode_fwd(cfg, x, theta)[:, 0]
    grid = theta[:, 0].reshape((N + 1,) * d)  # C order: last axis = dimension 0 (fastest)
    p = (x * np.float32(N)).astype(np.float64)  # the fp32-rounded scaled position
    ref = scipy.ndimage.map_coordinates(grid, [p[:, i] for i in reversed(range(d))], order=1, mode="nearest")
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("d", [1, 2, 3])
def test_affine_function_is_reproduced(d):
    # d-linear interpolation reproduces affine functions: theta(v) = a.v/N + c  =>  y(x) = a.(p/N) + c
    N = 24
    cfg = OracleConfig(d, 1, 1, (N + 1) ** d, N, N)
    lv = orc.levels(cfg)
    a = np.array([0.3, -1.7, 2.9])[:d]
    grids = np.meshgrid(*[np.arange(N + 1)] * d, indexing="ij")
    theta = np.zeros((lv.total, 1))
    for v in np.stack([g.ravel() for g in grids], axis=1):
        theta[orc.index(d, N + 1, cfg.T, True, v), 0] = float(a @ v) / N + 0.25
    x = np.random.default_rng(4).random((1000, d)).astype(np.float32)
    y = orc.encode_fwd(cfg, x, theta)[:, 0]
    p = (x * np.float32(N)).astype(np.float64)
    np.testing.assert_allclose(y, p @ a / N + 0.25, rtol=0, atol=1e-13)


def test_continuity_across_voxel_faces():
    # Section 5 (SDF discussion): the encoding is continuous; only its derivative jumps at faces
    cfg = OracleConfig(3, 8, 2, 1 << 12, 16, 256)
    lv, _, theta = _rand_cfg_inputs(cfg, 1, 6)
    rng = np.random.default_rng(7)
    for l in (0, 3, 7):
        N = int(lv.N[l])
        k = rng.integers(1, N, size=200)
        base = rng.random((200, 3)).astype(np.float32)
        lo, hi = base.copy(), base.copy()
        face = (k / N).astype(np.float32)
        lo[:, 1] = np.nextafter(face, np.float32(0))
        hi[:, 1] = face
        jump = np.abs(orc.encode_fwd(cfg, lo, theta) - orc.encode_fwd(cfg, hi, theta))
        assert jump.max() < 1e-3  # two adjacent fp32 positions; table values are O(1), N <= 256


def test_levels_are_independent_and_concatenated():
    # changing one level's table changes only that level's F output columns
    cfg = OracleConfig(3, 5, 2, 1 << 10, 4, 64)
    lv, x, theta = _rand_cfg_inputs(cfg, 200, 8)
    y0 = orc.encode_fwd(cfg, x, theta)
    for l in range(cfg.L):
        t2 = theta.copy()
        t2[int(lv.offset[l]):int(lv.offset[l]) + int(lv.size[l])] += 1.0
        diff = orc.encode_fwd(cfg, x, t2) - y0
        cols = np.zeros(cfg.L * cfg.F, bool)
        cols[l * cfg.F:(l + 1) * cfg.F] = True
        np.testing.assert_allclose(diff[:, cols], 1.0, atol=1e-12)
        assert (diff[:, ~cols] == 0).all()


def test_rejects_points_outside_unit_cube():
    cfg = OracleConfig(2, 2, 1, 64, 2, 4)
    theta = np.zeros((orc.levels(cfg).total, 1))
    for bad in (1.0, -0.1, np.nan, np.inf):
        with pytest.raises(ValueError):
            orc.encode_fwd(cfg, np.array([[0.5, bad]], np.float32), theta)


# ----------------------------------------------------------------------------- backward (Fig. 3 caption)

@pytest.mark.parametrize("interp", [0, 1])
@pytest.mark.parametrize("d,L,T,N_min,N_max", [(2, 4, 1 << 10, 4, 32), (3, 6, 1 << 9, 4, 64)])
def test_backward_is_adjoint_of_forward(d, L, T, N_min, N_max, interp):
    # y = J theta is linear in theta; the backward must be J^T:  <J v, g> = <v, J^T g>
    cfg = OracleConfig(d, L, 2, T, N_min, N_max, interp)
    lv, x, v = _rand_cfg_inputs(cfg, 700, 9)
    g = np.random.default_rng(10).standard_normal((700, L * 2))
    lhs = float((orc.encode_fwd(cfg, x, v) * g).sum())
    rhs = float((v * orc.encode_bwd(cfg, x, g)).sum())
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_backward_equals_dense_jacobian_transpose_bruteforce():
    # tiny case: build J column by column with unit tables, compare J^T g with the backward
    cfg = OracleConfig(2, 3, 2, 64, 2, 16)
    lv = orc.levels(cfg)
    assert lv.dense[0] and not lv.dense[-1]
    rng = np.random.default_rng(11)
    x = rng.random((50, 2)).astype(np.float32)
    g = rng.standard_normal((50, cfg.L * cfg.F))
    n = lv.total * cfg.F
    J = np.zeros((50 * cfg.L * cfg.F, n))
    for k in range(n):
        e = np.zeros(n)
        e[k] = 1.0
        J[:, k] = orc.encode_fwd(cfg, x, e.reshape(lv.total, cfg.F)).ravel()
    # each output is touched by exactly 2^d corners of its own level; the row sums are 1
    np.testing.assert_allclose(J.sum(axis=1), 1.0, atol=1e-14)
    dtheta = orc.encode_bwd(cfg, x, g)
    np.testing.assert_allclose(dtheta.ravel(), J.T @ g.ravel(), rtol=0, atol=1e-12)


def test_backward_finite_differences_of_a_loss():
    # loss = 0.5 |y|^2, dL/dy = y; central differences in theta (exact for a quadratic up to rounding)
    cfg = OracleConfig(2, 4, 2, 1 << 10, 4, 32)
    lv, x, theta = _rand_cfg_inputs(cfg, 64, 12)
    y = orc.encode_fwd(cfg, x, theta)
    grad = orc.encode_bwd(cfg, x, y)
    rng = np.random.default_rng(13)
    touched = np.argwhere(grad != 0)
    for e, f in touched[rng.choice(len(touched), 60, replace=False)]:
        h = 1e-4
        tp, tm = theta.copy(), theta.copy()
        tp[e, f] += h
        tm[e, f] -= h
        fd = (0.5 * (orc.encode_fwd(cfg, x, tp) ** 2).sum() - 0.5 * (orc.encode_fwd(cfg, x, tm) ** 2).sum()) / (2 * h)
        assert abs(fd - grad[e, f]) <= 1e-8 * max(1.0, abs(fd))


def test_backward_accumulates_into_given_buffer_and_sums_collisions():
    cfg = OracleConfig(2, 2, 1, 4, 8, 16)  # T = 4: heavy collisions on both (hashed) levels
    lv = orc.levels(cfg)
    assert not lv.dense.any() and lv.total == 8
    x = np.random.default_rng(14).random((300, 2)).astype(np.float32)
    g = np.ones((300, 2))
    dtheta = orc.encode_bwd(cfg, x, g)
    # every point distributes total weight 1 per level: sums are conserved (plain sum, no averaging)
    np.testing.assert_allclose(dtheta[:4].sum(), 300.0, atol=1e-10)
    np.testing.assert_allclose(dtheta[4:].sum(), 300.0, atol=1e-10)
    again = orc.encode_bwd(cfg, x, g, dtheta.copy())
    np.testing.assert_allclose(again, 2 * dtheta, atol=1e-10)


# ----------------------------------------------------------------------------- d(y)/d(x)

@pytest.mark.parametrize("interp", [0, 1])
def test_input_gradient_central_differences(interp):
    # power-of-two resolutions: x*N_l is exact in fp32, so along one axis inside a voxel the
    # d-linear encoding is exactly linear and central differences are exact up to rounding;
    # with the smoothstep it is a cubic in the fractional position and the stencil error is
    # h^2/6 * |third derivative| = h^2/6 * 12 N^3 |delta theta| (about 1e-2 here).
    cfg = OracleConfig(3, 4, 2, 1 << 9, 4, 32, interp)
    lv, _, theta = _rand_cfg_inputs(cfg, 1, 15)
    rng = np.random.default_rng(16)
    # positions k*2^-5 + off*2^-12 with off in [72,120): at least 8*2^-12 away from every voxel
    # face of every level, both for the plain grid (faces at multiples of 2^-5) and for the
    # half-voxel-shifted one (faces at odd multiples of 2^-6 = offset 64)
    x = ((rng.integers(0, 32, (80, 3)) * 128 + rng.integers(72, 120, (80, 3))) / 4096.0).astype(np.float32)
    g = rng.standard_normal((80, cfg.L * cfg.F))
    dx = orc.encode_bwd_input(cfg, x, theta, g)
    h = np.float32(2.0 ** -12)
    for j in range(3):
        xp, xm = x.copy(), x.copy()
        xp[:, j] += h
        xm[:, j] -= h
        fd = ((orc.encode_fwd(cfg, xp, theta) - orc.encode_fwd(cfg, xm, theta)) * g).sum(axis=1) / (2.0 * float(h))
        err = np.abs(fd - dx[:, j]).max()
        assert err <= (1e-9 if interp == 0 else 5e-2) * max(1.0, np.abs(fd).max()), err


def test_input_gradient_is_piecewise_constant_along_its_own_axis():
    # d-linear: d y / d x_j does not depend on x_j inside a voxel
    cfg = OracleConfig(3, 1, 2, 17 ** 3, 16, 16)
    lv, _, theta = _rand_cfg_inputs(cfg, 1, 17)
    g = np.ones((3, 2))
    x = np.array([[0.51, 0.3, 0.7], [0.53, 0.3, 0.7], [0.55, 0.3, 0.7]], np.float32)  # same voxel along x_0
    dx = orc.encode_bwd_input(cfg, x, theta, g)
    np.testing.assert_allclose(dx[:, 0], dx[0, 0], rtol=1e-12)
    assert np.ptp(dx[:, 1]) > 0  # but it does depend on x_0 for the other axes


# ----------------------------------------------------------------------------- smoothstep variant (Appendix A)

def test_smoothstep_closed_forms():
    # one level, d = 1, N = 8 (shifted grid: vertex k sits at x = (k - 0.5)/N)
    N = 8
    cfg = OracleConfig(1, 1, 1, 64, N, N, 1)
    lv = orc.levels(cfg)
    assert lv.dense[0] and lv.size[0] == N + 2
    theta = np.arange(N + 2, dtype=np.float64).reshape(-1, 1) ** 2
    # at vertices: exact table value
    k = np.arange(1, N + 1)
    xv = ((k - 0.5) / N).astype(np.float32).reshape(-1, 1)
    np.testing.assert_array_equal(orc.encode_fwd(cfg, xv, theta)[:, 0], theta[k, 0])
    # halfway between two vertices S(1/2) = 1/2: the mean of the two entries
    xm = (np.arange(1, N) / N).astype(np.float32)
    np.testing.assert_allclose(orc.encode_fwd(cfg, xm.reshape(-1, 1), theta)[:, 0],
                               0.5 * (theta[1:N, 0] + theta[2:N + 1, 0]), atol=1e-14)
    # quarter point: S(1/4) = 1/16 * (3 - 1/2) = 5/32
    xq = np.array([[(3 - 0.5 + 0.25) / N]], np.float32)
    np.testing.assert_allclose(orc.encode_fwd(cfg, xq, theta)[0, 0], theta[3, 0] * (1 - 5 / 32) + theta[4, 0] * 5 / 32,
                               atol=1e-14)
    # derivative vanishes at vertices (S'(0) = S'(1) = 0): the encoding is C^1
    np.testing.assert_allclose(orc.encode_bwd_input(cfg, xv, theta, np.ones((N, 1))), 0.0, atol=1e-12)
    # and equals S'(1/2) * N * (difference) = 1.5 N (theta[k+1] - theta[k]) halfway
    dmid = orc.encode_bwd_input(cfg, xm.reshape(-1, 1), theta, np.ones((N - 1, 1)))[:, 0]
    np.testing.assert_allclose(dmid, 1.5 * N * (theta[2:N + 1, 0] - theta[1:N, 0]), rtol=1e-13)


# ----------------------------------------------------------------------------- the entry every corner maps to

_PRIMES = (1, 2654435761, 805459861)


def _entry_bigint(v, verts, T, dense):
    """Section 3 / Eq. 4 for one integer vertex, in Python integers: the 1:1 map
    v_0 + v_1 V + v_2 V^2 on a coarse level, else XOR_i (v_i pi_i mod 2^32) mod T."""
    if dense:
        return sum(int(vi) * verts ** i for i, vi in enumerate(v))
    h = 0
    for i, vi in enumerate(v):
        h ^= (int(vi) * _PRIMES[i]) & 0xFFFFFFFF
    return h % T


@pytest.mark.parametrize("interp", [0, 1])
@pytest.mark.parametrize("d,L,T,N_min,N_max", [(1, 5, 40, 4, 300), (2, 6, 1 << 10, 4, 200), (3, 6, 1 << 12, 4, 100),
                                               (2, 5, 1000, 3, 97), (3, 5, 12345, 5, 80), (3, 16, 1 << 19, 16, 2048)])
def test_corner_entries_match_bigint_formulas_corner_by_corner(d, L, T, N_min, N_max, interp):
    # corner m is the upper corner along dimension i exactly when bit i of m is set (the order the
    # GPU library's debug call is compared in, bit for bit); the vertex it stands for is
    # floor(p) + bits with p = x N_l (+ 1/2 for Appendix A), evaluated here in fp32 by numpy
    cfg = OracleConfig(d, L, 2, T, N_min, N_max, interp)
    lv = orc.levels(cfg)
    assert lv.dense.any() and not lv.dense.all()
    x = np.random.default_rng(20 + d + 10 * interp).random((300, d)).astype(np.float32)
    for l in range(L):
        N, V = int(lv.N[l]), int(lv.N[l]) + 1 + interp
        assert int(lv.verts[l]) == V
        p = x * np.float32(N)
        if interp:
            p = p + np.float32(0.5)
        c0 = np.floor(p).astype(np.int64)
        idx, w = orc.indices(cfg, x, l)
        np.testing.assert_array_equal(w, p - np.floor(p))
        for b in range(len(x)):
            for m in range(1 << d):
                v = [int(c0[b, i]) + ((m >> i) & 1) for i in range(d)]
                assert int(idx[b, m]) == _entry_bigint(v, V, T, bool(lv.dense[l])), (l, b, m)
        assert int(idx.max()) < int(lv.size[l])


@pytest.mark.parametrize("interp", [0, 1])
@pytest.mark.parametrize("d", [1, 2, 3])
def test_forward_rebuilt_from_reported_entries_and_positions(d, interp):
    # sum_m weight_m theta[idx_m], with idx_m and the fractional positions as the oracle reports them and
    # the weights of Section 3 (Appendix A: S(w)) formed here, is the oracle's forward: the reported
    # entries are the ones the passes use, in the documented corner order
    cfg = OracleConfig(d, 5, 3, 1 << 9, 3, 150, interp)
    lv, x, theta = _rand_cfg_inputs(cfg, 400, 30 + d)
    y = orc.encode_fwd(cfg, x, theta)
    for l in range(cfg.L):
        idx, w = orc.indices(cfg, x, l)
        w = w.astype(np.float64)
        if interp:
            w = w * w * (3.0 - 2.0 * w)
        acc = np.zeros((len(x), cfg.F))
        for m in range(1 << d):
            wt = np.ones(len(x))
            for i in range(d):
                wt = wt * (w[:, i] if (m >> i) & 1 else 1.0 - w[:, i])
            acc += wt[:, None] * theta[int(lv.offset[l]) + idx[:, m].astype(np.int64)]
        np.testing.assert_allclose(y[:, l * cfg.F:(l + 1) * cfg.F], acc, rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- Appendix A on 1:1 levels, d >= 2

@pytest.mark.parametrize("d,N", [(2, 8), (3, 4), (3, 8)])
def test_shifted_grid_vertex_exactness_and_one_to_one_map(d, N):
    # Appendix A shifts every level by half a voxel: vertex k of the shifted grid sits at
    # x = (k - 1/2)/N_l (exact in fp32 for a power-of-two N_l), k = 0 .. N_l+1.  At such a point the
    # output is the table entry of that vertex (S(0) = 0), and on a 1:1 level the entry of vertex v is
    # v_0 + v_1 (N_l+2) + v_2 (N_l+2)^2: every entry holds its own index here, so any other stride shows.
    V = N + 2
    cfg = OracleConfig(d, 1, 1, V ** d, N, N, 1)
    lv = orc.levels(cfg)
    assert lv.dense[0] and int(lv.size[0]) == V ** d and int(lv.verts[0]) == V
    theta = np.arange(V ** d, dtype=np.float64).reshape(-1, 1)
    grids = np.meshgrid(*[np.arange(1, N + 1)] * d, indexing="ij")  # vertices with x = (k - 1/2)/N in [0,1)
    k = np.stack([g.ravel() for g in grids], axis=1)
    x = ((k - 0.5) / N).astype(np.float32)
    y = orc.encode_fwd(cfg, x, theta)[:, 0]
    expect = sum(k[:, i] * V ** i for i in range(d))
    np.testing.assert_array_equal(y, expect.astype(np.float64))
    # every voxel of the shifted grid, one point each: the corners seen cover all (N+2)^d vertices and
    # the map vertex -> entry is a bijection onto 0 .. (N+2)^d - 1
    grids = np.meshgrid(*[np.arange(0, N + 1)] * d, indexing="ij")
    c = np.stack([g.ravel() for g in grids], axis=1)
    xv = np.where(c == 0, 0.1 / N, (c - 0.25) / N).astype(np.float32)  # p = x N + 1/2 lies inside voxel c
    assert (xv < 1).all()
    idx, w = orc.indices(cfg, xv, 0)
    seen = {}
    for b in range(len(c)):
        for m in range(1 << d):
            v = tuple(int(c[b, i]) + ((m >> i) & 1) for i in range(d))
            assert seen.setdefault(v, int(idx[b, m])) == int(idx[b, m])
    assert len(seen) == V ** d and sorted(seen.values()) == list(range(V ** d))
    for v, e in seen.items():
        assert e == sum(vi * V ** i for i, vi in enumerate(v))


def test_shifted_grid_dense_criterion_uses_its_own_vertex_count():
    # (N_l+2)^d <= T decides 1:1 for Appendix A's grid: N = 15, d = 2: 16^2 = 256 fits T = 256 without
    # the shift, 17^2 = 289 does not with it
    assert orc.levels(OracleConfig(2, 1, 1, 256, 15, 15, 0)).dense[0]
    assert not orc.levels(OracleConfig(2, 1, 1, 256, 15, 15, 1)).dense[0]
    assert orc.levels(OracleConfig(2, 1, 1, 289, 15, 15, 1)).dense[0]


@pytest.mark.parametrize("d", [2, 3])
def test_shifted_grid_backward_puts_unit_mass_on_the_vertex_entry(d):
    # the backward pass of a point that sits on a vertex of the shifted grid adds dL/dy to that
    # vertex's entry and to no other (weights 1 and 0)
    N, V = 8, 10
    cfg = OracleConfig(d, 1, 1, V ** d, N, N, 1)
    k = np.array([[3, 7, 1][:d]])
    x = ((k - 0.5) / N).astype(np.float32)
    g = orc.encode_bwd(cfg, x, np.array([[2.5]]))
    e = sum(int(k[0, i]) * V ** i for i in range(d))
    assert g[e, 0] == 2.5 and np.count_nonzero(g) == 1
