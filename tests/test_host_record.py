"""The record of the sorted backward pass and the fixed-point product of its accumulate pass
(csrc/bwd_record.hpp), compiled for the host by tests/record_check.hip and checked without a GPU:
what is packed comes back as the format says, the weights move by no more than the 2^-23 that the
parity tests allow for them, and the product is the exact one, rounded once, ties to even."""
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
    so.record_roundtrip.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int, P, P, P, P, P, ctypes.c_int,
                                    ctypes.c_uint32, ctypes.c_uint32, ctypes.c_double, P, P, P, P, P]
    so.fixed_products.restype = None
    so.fixed_products.argtypes = [ctypes.c_uint32, P, P, P]
    return so


def roundtrip(lib, F, half, la, k, wf0, wrow, g, dense, cmask, xmask, scale):
    n = len(la)
    words = ctypes.c_uint32(0)
    out_la, out_lb = np.zeros(n, np.uint32), np.zeros(n, np.uint32)
    out_wf0, out_G = np.zeros(n, np.float32), np.zeros((n, F), np.float64)
    arrs = [np.ascontiguousarray(a) for a in (la.astype(np.uint32), k.astype(np.uint32), wf0.astype(np.float32),
                                              wrow.astype(np.float32), g.astype(np.float32))]
    st = lib.record_roundtrip(n, F, int(half), *(a.ctypes.data for a in arrs), int(dense), cmask, xmask, scale,
                              ctypes.addressof(words), out_la.ctypes.data, out_lb.ctypes.data,
                              out_wf0.ctypes.data, out_G.ctypes.data)
    assert st == 0
    return words.value, out_la, out_lb, out_wf0, out_G


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
    k = rng.integers(0, 13, n)
    wf0 = rng.random(n, dtype=np.float32)
    wrow = rng.random(n, dtype=np.float32)
    # the ends of both ranges, and fractions that are multiples of 2^-23 (what a scaled coordinate >= 1 gives)
    wf0[:4] = [0.0, np.float32(1 - 2.0 ** -24), 0.5, 2.0 ** -24]
    wrow[:4] = [0.0, 1.0, np.float32(1 - 2.0 ** -24), 2.0 ** -25]
    wf0[4:1000] = (rng.integers(0, 1 << 23, 996) * 2.0 ** -23).astype(np.float32)
    g = rng.standard_normal((n, F)).astype(np.float16 if half else np.float32)
    scale = 2.0 ** 17
    words, out_la, out_lb, out_wf0, out_G = roundtrip(lib, F, half, la, k, wf0, wrow, g, dense, cmask, xmask, scale)
    assert words == 2 + (F * (2 if half else 4) + 3) // 4
    np.testing.assert_array_equal(out_la, la)
    lb = (la + 1) & cmask if dense else la ^ (((2 << k) - 1) & xmask)
    np.testing.assert_array_equal(out_lb, lb)
    # position along dimension 0: units of 2^-23, at most 2^-24 off, exact for multiples of 2^-23
    assert np.abs(out_wf0.astype(np.float64) - wf0.astype(np.float64)).max() <= 2.0 ** -24
    np.testing.assert_array_equal(out_wf0[4:1000], wf0[4:1000])
    assert out_wf0.max() < 1.0
    # weight of the other dimensions: units of 2^-24 (ties to even), times dL/dy, times the scale: exact
    q = np.rint(wrow.astype(np.float64) * 2.0 ** 24)
    assert np.abs(q * 2.0 ** -24 - wrow).max() <= 2.0 ** -25
    np.testing.assert_array_equal(out_G, (q * (scale * 2.0 ** -24))[:, None] * g.astype(np.float64))
    assert out_G[0].tolist() == [0.0] * F and (out_G[1] == scale * g[1].astype(np.float64)).all()
    # the two corner weights of the pair move by no more than 2^-23 in all
    w_up, w_lo = wf0.astype(np.float64) * wrow, (1.0 - wf0.astype(np.float64)) * wrow
    r_up, r_lo = out_wf0.astype(np.float64) * q * 2.0 ** -24, (1.0 - out_wf0.astype(np.float64)) * q * 2.0 ** -24
    assert (np.abs(r_up - w_up) + np.abs(r_lo - w_lo)).max() <= 2.0 ** -23


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
