"""Pins of the network oracle (paper Section 4, "Architecture": two hidden layers of 64 neurons,
ReLU, linear output) against things other than itself: integer arithmetic done with Python ints,
hand-built networks with known outputs, a library evaluation (torch, fp64) where no rounding
can occur, and the rounding points themselves."""
import numpy as np
import torch

from oracle import hashgrid_oracle as orc
from oracle import mlp_oracle as mlp


def _int_net(rng, n_in, n_out, lo=-2, hi=3):
    return (rng.integers(lo, hi, (64, n_in)), rng.integers(lo, hi, (64, 64)), rng.integers(lo, hi, (n_out, 64)))


def test_small_integers_match_exact_integer_arithmetic():
    # every intermediate value is an integer below 2048 in magnitude: exactly representable in half
    # precision, so no rounding anywhere, and the result must equal big-integer arithmetic
    rng = np.random.default_rng(0)
    n_in, n_out, B = 32, 3, 17
    W1 = rng.integers(-1, 2, (64, n_in)) * (rng.random((64, n_in)) < 0.2)
    W2 = rng.integers(-1, 2, (64, 64)) * (rng.random((64, 64)) < 0.1)
    W3 = rng.integers(-3, 4, (n_out, 64))
    y = rng.integers(-3, 4, (B, n_in))
    out = mlp.mlp_fwd(y, W1, W2, W3)
    for b in range(B):
        h1 = [max(sum(int(W1[i, k]) * int(y[b, k]) for k in range(n_in)), 0) for i in range(64)]
        assert max(h1) < 2048
        h2 = [max(sum(int(W2[i, k]) * h1[k] for k in range(64)), 0) for i in range(64)]
        assert max(h2) < 2048
        ref = [sum(int(W3[i, k]) * h2[k] for k in range(64)) for i in range(n_out)]
        assert [int(v) for v in out[b]] == ref and (out[b] == np.round(out[b])).all()


def test_hand_built_network_selects_and_rectifies():
    # neuron i of layer 1 copies input i (i < n_in), layer 2 copies layer 1, output 0 sums the first
    # n_in neurons, output 1 takes neuron 0 negated: ReLU must clip negative inputs and only them
    n_in = 16
    W1 = np.zeros((64, n_in)); W1[np.arange(n_in), np.arange(n_in)] = 1
    W2 = np.eye(64)
    W3 = np.zeros((2, 64)); W3[0, :n_in] = 1; W3[1, 0] = -1
    y = np.array([[1.5, -2.0] + [0.25] * 14, [-1.0] * 16, [0.0] * 16])
    out = mlp.mlp_fwd(y, W1, W2, W3)
    np.testing.assert_array_equal(out, [[1.5 + 14 * 0.25, -1.5], [0.0, 0.0], [0.0, 0.0]])


def test_row_is_neuron_not_input():
    # a transposed weight matrix must change the answer: W1[i, k] multiplies input k into neuron i
    W1 = np.zeros((64, 64)); W1[5, 9] = 1.0
    W2 = np.eye(64); W3 = np.eye(64)
    y = np.zeros((1, 64)); y[0, 9] = 2.0
    out = mlp.mlp_fwd(y, W1, W2, W3)
    assert out[0, 5] == 2.0 and out[0, 9] == 0.0 and out.sum() == 2.0


def test_matches_library_evaluation_when_nothing_rounds():
    # multiples of 1/8 with small integer weights: all intermediates are exactly representable in
    # half precision, so the rounding points are the identity and torch's fp64 evaluation must agree
    rng = np.random.default_rng(3)
    W1 = rng.integers(-1, 2, (64, 32)) * (rng.random((64, 32)) < 0.15)
    W2 = rng.integers(-1, 2, (64, 64)) * (rng.random((64, 64)) < 0.08)
    W3 = rng.integers(-2, 3, (4, 64))
    y = rng.integers(-8, 9, (50, 32)) / 8.0
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    h = torch.relu(torch.nn.functional.linear(t(y), t(W1)))
    h = torch.relu(torch.nn.functional.linear(h, t(W2)))
    ref = torch.nn.functional.linear(h, t(W3)).numpy()
    assert np.abs(ref).max() > 0
    np.testing.assert_array_equal(mlp.mlp_fwd(y, W1, W2, W3), ref)


def test_rounding_points_are_half_precision_to_nearest_even():
    # input: 1 + 2^-11 is a tie between 1 and 1 + 2^-10 -> 1 (even); 1 + 3*2^-11 -> 1 + 2^-9 (even)
    W1 = np.zeros((64, 8)); W1[0, 0] = 1.0; W1[1, 1] = 1.0
    W2 = np.eye(64); W3 = np.eye(64)[:2]
    y = np.zeros((1, 8)); y[0, 0] = 1 + 2.0 ** -11; y[0, 1] = 1 + 3 * 2.0 ** -11
    out = mlp.mlp_fwd(y, W1, W2, W3)
    np.testing.assert_array_equal(out[0], [1.0, 1 + 2.0 ** -9])
    # each hidden layer rounds what it stores: 0.7 becomes 0.7001953125 (= 2868 * 2^-12) after layer 1 ...
    W1 = np.zeros((64, 8)); W1[0, 0] = 0.7   # weights keep whatever precision they are given in
    y = np.zeros((1, 8)); y[0, 0] = 1.0
    out = mlp.mlp_fwd(y, W1, np.eye(64), np.eye(64)[:1])
    assert out[0, 0] == 2868 * 2.0 ** -12 and out[0, 0] != 0.7
    # ... and after layer 2
    W1 = np.zeros((64, 8)); W1[0, 0] = 1.0
    W2 = np.zeros((64, 64)); W2[0, 0] = 0.7
    out = mlp.mlp_fwd(y, W1, W2, np.eye(64)[:1])
    assert out[0, 0] == 2868 * 2.0 ** -12
    # the output layer is not rounded
    W3 = np.zeros((1, 64)); W3[0, 0] = 1 / 3
    out = mlp.mlp_fwd(np.eye(8)[:1], np.eye(64)[:, :8], np.eye(64), W3)
    assert out[0, 0] == 1 / 3


def test_encoding_feeds_the_network():
    # a one-level dense grid whose entries are all 0.5: the encoding returns 0.5 everywhere
    # (weights sum to 1), so the network sees a constant input
    cfg = orc.OracleConfig(2, 4, 2, 1 << 10, 4, 32)
    lv = orc.levels(cfg)
    theta = np.full((lv.total, 2), 0.5)
    x = np.random.default_rng(1).random((9, 2)).astype(np.float32) * 0.99
    W1 = np.zeros((64, 8)); W1[0, :] = 1.0
    out = mlp.encode_mlp_fwd(cfg, x, theta, W1, np.eye(64), np.eye(64)[:1])
    np.testing.assert_allclose(out[:, 0], 4.0, rtol=0, atol=1e-12)


def test_magnitude_bound_dominates_the_output():
    rng = np.random.default_rng(5)
    W1, W2, W3 = (rng.standard_normal(s) for s in ((64, 32), (64, 64), (3, 64)))
    y = rng.standard_normal((20, 32))
    assert (np.abs(mlp.mlp_fwd(y, W1, W2, W3)) <= mlp.magnitude_bound(y, W1, W2, W3) * (1 + 1e-2)).all()


# ----------------------------------------------------------------------------- backward pass of the network

def _torch_grads(y, W1, W2, W3, dout):
    t = [torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for a in (y, W1, W2, W3)]
    out = torch.relu(torch.relu(t[0] @ t[1].T) @ t[2].T) @ t[3].T
    out.backward(torch.tensor(np.asarray(dout, dtype=np.float64)))
    return [a.grad.numpy() for a in t]


def test_backward_matches_library_autograd_without_rounding():
    rng = np.random.default_rng(40)
    B, n_in, n_out = 50, 32, 4
    y = rng.standard_normal((B, n_in))
    W1, W2, W3 = rng.standard_normal((64, n_in)) * 0.3, rng.standard_normal((64, 64)) * 0.2, rng.standard_normal((n_out, 64))
    dout = rng.standard_normal((B, n_out))
    got = mlp.mlp_bwd(y, W1, W2, W3, dout, rounding=False)
    for g, ref in zip(got, _torch_grads(y, W1, W2, W3, dout)):
        np.testing.assert_allclose(g, ref, rtol=1e-12, atol=1e-12)


def test_backward_with_rounding_equals_autograd_where_nothing_rounds():
    # small integers and multiples of 1/8 everywhere: every value the backward pass rounds to half
    # precision is exactly representable, so the rounding points are the identity
    rng = np.random.default_rng(41)
    B, n_in, n_out = 24, 16, 2
    W1 = rng.integers(-1, 2, (64, n_in)) * (rng.random((64, n_in)) < 0.2)
    W2 = rng.integers(-1, 2, (64, 64)) * (rng.random((64, 64)) < 0.1)
    W3 = rng.integers(-2, 3, (n_out, 64))
    y = rng.integers(-8, 9, (B, n_in)) / 8.0
    dout = rng.integers(-4, 5, (B, n_out)) / 4.0
    got = mlp.mlp_bwd(y, W1, W2, W3, dout)
    ref = _torch_grads(y, W1, W2, W3, dout)
    for g, r in zip(got, ref):
        np.testing.assert_array_equal(g, r)
    assert np.abs(ref[0]).max() > 0 and np.abs(ref[1]).max() > 0


def test_backward_finite_differences_of_a_linear_loss():
    # loss = sum(out * c): dL/dout = c; central differences in single weights and inputs, on the
    # rounding-free network, at points no perturbation moves across a ReLU kink (checked)
    rng = np.random.default_rng(42)
    B, n_in, n_out = 6, 8, 3
    y = rng.standard_normal((B, n_in))
    Ws = [rng.standard_normal((64, n_in)) * 0.5, rng.standard_normal((64, 64)) * 0.2, rng.standard_normal((n_out, 64))]
    c = rng.standard_normal((B, n_out))
    grads = mlp.mlp_bwd(y, *Ws, c, rounding=False)

    def loss(yy, ws):
        h1 = np.maximum(yy @ ws[0].T, 0.0)
        h2 = np.maximum(h1 @ ws[1].T, 0.0)
        return float(((h2 @ ws[2].T) * c).sum()), (h1 > 0, h2 > 0)

    _, pattern = loss(y, Ws)
    h = 1e-6
    checked = 0
    for which in range(4):
        arr = y if which == 0 else Ws[which - 1]
        for _ in range(12):
            i, j = rng.integers(0, arr.shape[0]), rng.integers(0, arr.shape[1])
            plus, minus = arr.copy(), arr.copy()
            plus[i, j] += h
            minus[i, j] -= h
            args_p = (plus, Ws) if which == 0 else (y, [plus if k == which - 1 else Ws[k] for k in range(3)])
            args_m = (minus, Ws) if which == 0 else (y, [minus if k == which - 1 else Ws[k] for k in range(3)])
            lp, pp = loss(*args_p)
            lm, pm = loss(*args_m)
            if not all((a == b).all() and (a == p0).all() for a, b, p0 in zip(pp, pm, pattern)):
                continue  # a kink lies inside the stencil
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grads[which][i, j]) <= 1e-6 * max(1.0, abs(fd))
            checked += 1
    assert checked > 30


def test_backward_of_a_hand_built_network():
    # layer 1 copies input k to neuron k, layer 2 copies, output 0 sums neurons 0..n_in-1:
    # dL/dy_k = dL/dout_0 where y_k > 0, else 0 (ReLU closed); dW3[0, k] = sum_b dout_0 * relu(y_k)
    n_in = 8
    W1 = np.zeros((64, n_in)); W1[np.arange(n_in), np.arange(n_in)] = 1
    W2 = np.eye(64)
    W3 = np.zeros((1, 64)); W3[0, :n_in] = 1
    y = np.array([[1.0, -1.0, 2.0, 0.0, 0.5, -3.0, 4.0, 0.25], [-1.0] * 8])
    dout = np.array([[2.0], [5.0]])
    dy, dW1, dW2, dW3 = mlp.mlp_bwd(y, W1, W2, W3, dout)
    np.testing.assert_array_equal(dy, [[2, 0, 2, 0, 2, 0, 2, 2], [0] * 8])  # nothing passes at y = 0 or below
    np.testing.assert_array_equal(dW3[0, :n_in], 2.0 * np.maximum(y[0], 0))
    assert dW3[0, n_in:].sum() == 0
    # dW1[i, k] = g1[i] * y[k] summed over the batch: neuron i is open only where y_i > 0
    expect = np.zeros((64, n_in))
    for i in range(n_in):
        if y[0, i] > 0:
            expect[i] = 2.0 * y[0]
    np.testing.assert_array_equal(dW1, expect)


def test_backward_rounding_points():
    # the upstream gradient becomes a half-precision operand: 1 + 2^-12 rounds to 1; hidden gradients too
    W1 = np.zeros((64, 8)); W1[0, 0] = 1
    W2 = np.zeros((64, 64)); W2[0, 0] = 1
    W3 = np.zeros((1, 64)); W3[0, 0] = 1 + 2.0 ** -10      # representable in half precision
    y = np.zeros((1, 8)); y[0, 0] = 1.0
    dout = np.array([[1.0 + 2.0 ** -12]])
    dy, dW1, dW2, dW3 = mlp.mlp_bwd(y, W1, W2, W3, dout)
    assert dW3[0, 0] == 1.0                                  # half(dout) * h2
    # g2 = half(1 * (1 + 2^-10)) = 1 + 2^-10 exactly; g1 = half(g2 * 1) the same; dy = g1 * W1
    assert dy[0, 0] == 1 + 2.0 ** -10
    dy2, *_ = mlp.mlp_bwd(y, W1, W2, W3, dout, rounding=False)
    assert dy2[0, 0] == (1.0 + 2.0 ** -12) * (1 + 2.0 ** -10)
