"""The record of the sorted backward pass and the fixed-point product of its accumulate pass
(csrc/bwd_record.hpp), compiled for the host by tests/record_check.hip and checked without a GPU:
what is packed comes back as the format says, the weights keep the relative precision the header
promises (2^-20 for the product over the other dimensions, exact along dimension 0 from the second
voxel on, 2^-17 in the first voxel), and the product is the exact one, rounded once, ties to even."""
import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np
import pytest

from paper_2201_05989_amd.build import CSRC, INCLUDE, hipcc

HERE = os.path.dirname(os.path.abspath(__file__))
P = ctypes.c_void_p


@pytest.fixture(scope="module")
def lib(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("record") / "librecord_check.so")
    cmd = [hipcc(), "--cuda-host-only", "-O2", "-ffp-contract=off", "-fPIC", "-shared", f"-I{INCLUDE}", f"-I{CSRC}",
           os.path.join(HERE, "record_check.hip"), "-o", out]
    subprocess.run(cmd, check=True, capture_output=True)
    so = ctypes.CDLL(out)
    so.record_roundtrip.restype = ctypes.c_int
    so.record_roundtrip.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int, P, P, P, P, P, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_uint32, ctypes.c_uint32, ctypes.c_double, P, P, P, P, P, P]
    so.fixed_products.restype = None
    so.fixed_products.argtypes = [ctypes.c_uint32, P, P, P]
    return so


def roundtrip(lib, F, half, la, k, wf0, wrow, g, dense, cmask, xmask, scale, smooth=False):
    n = len(la)
    words = ctypes.c_uint32(0)
    out_la, out_lb = np.zeros(n, np.uint32), np.zeros(n, np.uint32)
    out_wlo, out_wup, out_G = np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros((n, F), np.float64)
    arrs = [np.ascontiguousarray(a) for a in (la.astype(np.uint32), k.astype(np.uint32), wf0.astype(np.float32),
                                              wrow.astype(np.float32), g.astype(np.float32))]
    st = lib.record_roundtrip(n, F, int(half), *(a.ctypes.data for a in arrs), int(dense), int(smooth), cmask, xmask, scale,
                              ctypes.addressof(words), out_la.ctypes.data, out_lb.ctypes.data,
                              out_wlo.ctypes.data, out_wup.ctypes.data, out_G.ctypes.data)
    assert st == 0
    return words.value, out_la, out_lb, out_wlo, out_wup, out_G


def small_float(w, mbits, low):
    """A weight rounded to `mbits` mantissa bits (half up), 0 below 2^(low - 127): the format's definition."""
    w = np.asarray(w, np.float32)
    b = w.view(np.uint32).astype(np.uint64) + (1 << (22 - mbits))
    b = (b >> (23 - mbits)) << (23 - mbits)
    out = b.astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where((b >> 23) < low, 0.0, out)


@pytest.mark.parametrize("F", [1, 2, 4, 8])
@pytest.mark.parametrize("half", [True, False])
@pytest.mark.parametrize("dense", [True, False])
def test_record_round_trip(lib, F, half, dense):
    rng = np.random.default_rng(F * 4 + half * 2 + dense)
    n = 20000
    cap = 2048 if F == 8 else 4096
    cmask = cap - 1
    xmask = int(rng.choice([cmask, 255, 0]))            # a hashed table smaller than a chunk wraps the step
    la = rng.integers(0, (xmask + 1) if not dense else cap - 1, n)
    k = rng.integers(0, 15, n)                          # (rows_of caps the trailing ones at 14)
    wf0 = rng.random(n, dtype=np.float32)
    # weights of every size: products of one or two fractions, some of them tiny
    wrow = (rng.random(n, dtype=np.float32) * rng.random(n, dtype=np.float32) ** rng.integers(0, 12, n)).astype(np.float32)
    # the ends of both ranges, and fractions that are multiples of 2^-23 (what a scaled coordinate >= 1 gives)
    wf0[:4] = [0.0, np.float32(1 - 2.0 ** -23), 0.5, 2.0 ** -23]
    wrow[:6] = [0.0, 1.0, np.float32(1 - 2.0 ** -24), 2.0 ** -25, 2.0 ** -62, 2.0 ** -63]
    wf0[4:] = (rng.integers(0, 1 << 23, n - 4) * 2.0 ** -23).astype(np.float32)
    g = rng.standard_normal((n, F)).astype(np.float16 if half else np.float32)
    scale = 2.0 ** 17
    words, out_la, out_lb, out_wlo, out_wup, out_G = roundtrip(lib, F, half, la, k, wf0, wrow, g, dense, cmask, xmask, scale)
    assert words == 2 + (F * (2 if half else 4) + 3) // 4
    np.testing.assert_array_equal(out_la, la)
    lb = (la + 1) & cmask if dense else la ^ (((2 << k) - 1) & xmask)
    np.testing.assert_array_equal(out_lb, lb)
    # position along dimension 0 from the second voxel on: a multiple of 2^-23, kept exactly, both weights exact
    np.testing.assert_array_equal(out_wup, wf0)
    np.testing.assert_array_equal(out_wlo.astype(np.float64), 1.0 - wf0.astype(np.float64))
    # weight of the other dimensions: a small float of 19 mantissa bits, times dL/dy, times the scale: exact
    q = small_float(wrow, 19, 65)
    big = wrow >= 2.0 ** -62
    assert (np.abs(q[big] - wrow[big]) <= 2.0 ** -20 * wrow[big]).all() and (q[~big] == 0).all()
    np.testing.assert_array_equal(out_G, (q * scale)[:, None] * g.astype(np.float64))
    assert out_G[0].tolist() == [0.0] * F and (out_G[1] == scale * g[1].astype(np.float64)).all()
    assert (out_G[4] == scale * 2.0 ** -62 * g[4].astype(np.float64)).all() and (out_G[5] == 0).all()


@pytest.mark.parametrize("smooth", [False, True])
@pytest.mark.parametrize("dense", [True, False])
def test_record_of_the_first_voxel_keeps_both_weights_to_relative_precision(lib, dense, smooth):
    # k = 15: the scaled coordinate along dimension 0 is below 1, its fraction is any float; the record
    # then holds the smaller of the pair's two weights as a small float of 16 mantissa bits
    rng = np.random.default_rng(21 + dense)
    n = 20000
    cmask = xmask = 4095
    la = rng.integers(0, 4095, n)
    k = np.full(n, 15)
    wf0 = (rng.random(n, dtype=np.float32) * np.float32(2.0) ** -rng.integers(0, 66, n).astype(np.float32)).astype(np.float32)
    wf0[n // 2:] = np.float32(1.0) - wf0[n // 2:]       # and fractions close to 1 (the smoothstep variant's first voxel)
    wf0 = np.minimum(wf0, np.float32(1 - 2.0 ** -24))
    wf0[:5] = [0.0, 0.5, np.float32(1 - 2.0 ** -24), 2.0 ** -63, 2.0 ** -65]
    wrow = np.ones(n, np.float32)
    g = np.ones((n, 2), np.float32)
    _, out_la, out_lb, out_wlo, out_wup, _ = roundtrip(lib, 2, False, la, k, wf0, wrow, g, dense, cmask, xmask, 1.0, smooth)
    np.testing.assert_array_equal(out_la, la)
    np.testing.assert_array_equal(out_lb, (la + 1) & cmask if dense else la ^ 1)  # the coordinate is 0: k = 0
    up, lo = wf0.astype(np.float64), 1.0 - wf0.astype(np.float64)
    if smooth:  # Appendix A: the first-voxel form holds the final weights S(w), S(1 - w)
        up, lo = up * up * (3 - 2 * up), lo * lo * (3 - 2 * lo)
    small = np.minimum(up, lo)
    ok = small >= 2.0 ** -63
    for got, want in ((out_wup.astype(np.float64), up), (out_wlo.astype(np.float64), lo)):
        assert (np.abs(got[ok] - want[ok]) <= (2.0 ** -17 + 3e-7 * smooth) * want[ok] + 2.0 ** -25 * (want[ok] > 0.5)).all()
        assert (np.abs(got[~ok] - want[~ok]) <= 2.0 ** -63).all()
    assert out_wup[0] == 0.0 and out_wlo[0] == 1.0 and out_wup[1] == 0.5 and out_wlo[1] == 0.5
    if not smooth:
        assert out_wup[3] == np.float32(2.0 ** -63) and out_wup[4] == 0.0


def test_fixed_product_is_the_exact_product_rounded_once(lib):
    rng = np.random.default_rng(9)
    n = 4000
    w = rng.random(n, dtype=np.float32)
    G = rng.standard_normal(n) * 2.0 ** rng.integers(0, 50, n)
    G = np.clip(G, -(2.0 ** 50), 2.0 ** 50)
    # exact ties: half of an odd integer, both signs; zero; the largest magnitude served
    w[:6] = [0.5, 0.5, 0.5, 0.5, 0.0, 1.0]
    G[:6] = [3.0, 5.0, -3.0, -5.0, 123.0, 2.0 ** 51 - 1]
    out = np.zeros(n, np.int64)
    lib.fixed_products(n, w.ctypes.data, G.ctypes.data, out.ctypes.data)
    assert out[:6].tolist() == [2, 2, -2, -2, 0, 2 ** 51 - 1]
    for i in range(n):
        exact = Fraction(float(w[i])) * Fraction(float(G[i]))
        assert out[i] == round(exact)  # Python rounds a Fraction to the nearest integer, ties to even
