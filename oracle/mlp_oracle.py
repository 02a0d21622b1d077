"""CPU oracle of the small network that follows the encoding (paper Section 4, "Architecture":
two hidden layers of 64 neurons, ReLU on the hidden layers, a linear output layer), evaluated on
the encoding's output.  TEST INFRASTRUCTURE ONLY: the test-suite and the benchmark's CPU leg use
it; the GPU library never does.

Arithmetic: plain numpy in fp64, one matrix product per layer, in the paper's order.  The
readings that the paper leaves open are where values are rounded: the encoding's output and the
two hidden activations are rounded to half precision (round to nearest even), as stored by a
network that runs in half precision (Section 4, "Performance considerations": half-precision
arithmetic with full-precision accumulation is not spelled out; the GPU path accumulates each
dot product in fp32); the output layer's result is left in full precision.
"""
from __future__ import annotations

import numpy as np

from . import hashgrid_oracle as orc

N_HIDDEN = 64


def _half(a: np.ndarray) -> np.ndarray:
    """Round to the nearest fp16 (ties to even), returned as fp64."""
    return a.astype(np.float16).astype(np.float64)


def mlp_fwd(y, W1, W2, W3):
    """out [B, n_out] fp64 from y [B, n_in]; W1 [64, n_in], W2 [64, 64], W3 [n_out, 64] (row = neuron)."""
    y = _half(np.asarray(y, dtype=np.float64))
    W1, W2, W3 = (np.asarray(w).astype(np.float64) for w in (W1, W2, W3))
    assert W1.shape == (N_HIDDEN, y.shape[1]) and W2.shape == (N_HIDDEN, N_HIDDEN) and W3.shape[1] == N_HIDDEN
    h1 = _half(np.maximum(y @ W1.T, 0.0))
    h2 = _half(np.maximum(h1 @ W2.T, 0.0))
    return h2 @ W3.T


def encode_mlp_fwd(cfg: orc.OracleConfig, x, theta, W1, W2, W3):
    """The encoding (Section 3) followed by the network (Section 4): out [B, n_out] fp64."""
    return mlp_fwd(orc.encode_fwd(cfg, x, theta), W1, W2, W3)


def magnitude_bound(y, W1, W2, W3):
    """|W3| (|W2| (|W1| |y|)): what a relative perturbation of the activations is measured against."""
    a = np.abs(np.asarray(y, dtype=np.float64)) @ np.abs(np.asarray(W1, dtype=np.float64)).T
    a = a @ np.abs(np.asarray(W2, dtype=np.float64)).T
    return a @ np.abs(np.asarray(W3, dtype=np.float64)).T


def mlp_bwd(y, W1, W2, W3, dout, rounding: bool = True):
    """Backward pass of the network above (chain rule through the three layers of Section 4,
    "Architecture"; ReLU passes the gradient where its output is positive, nothing at 0).
    Returns (dy [B, n_in], dW1 [64, n_in], dW2 [64, 64], dW3 [n_out, 64]) in fp64, the weight
    gradients summed over the batch.

    The forward values are recomputed as mlp_fwd computes them.  Readings, where the paper is
    silent: a network that runs in half precision keeps its backward operands in half precision
    too, so the upstream gradient dL/dout and the two hidden-layer gradients are rounded to half
    (nearest even) where they become operands of the next product, exactly as the activations are
    on the way forward; roundings are treated as the identity by the chain rule; products
    accumulate in full precision; dy and the weight gradients are left in full precision.
    rounding=False drops every rounding (forward ones too): the plain fp64 network, which finite
    differences and a library's autograd can check."""
    r = _half if rounding else (lambda a: a)
    y = r(np.asarray(y, dtype=np.float64))
    W1, W2, W3 = (np.asarray(w).astype(np.float64) for w in (W1, W2, W3))
    h1 = r(np.maximum(y @ W1.T, 0.0))
    h2 = r(np.maximum(h1 @ W2.T, 0.0))
    g3 = r(np.asarray(dout, dtype=np.float64))        # dL/dout                     [B, n_out]
    dW3 = g3.T @ h2
    g2 = r((g3 @ W3) * (h2 > 0))                      # dL/d(pre-activation 2)      [B, 64]
    dW2 = g2.T @ h1
    g1 = r((g2 @ W2) * (h1 > 0))                      # dL/d(pre-activation 1)      [B, 64]
    dW1 = g1.T @ y
    dy = g1 @ W1
    return dy, dW1, dW2, dW3


def bwd_magnitudes(y, W1, W2, W3, dout):
    """Sums of absolute values along the same chains, for error bounds: (|dy|-bound [B, n_in],
    |dW1|, |dW2|, |dW3| bounds), every product taken with absolute values and every ReLU open."""
    y = np.abs(np.asarray(y, dtype=np.float64))
    A1, A2, A3 = (np.abs(np.asarray(w).astype(np.float64)) for w in (W1, W2, W3))
    h1 = y @ A1.T
    h2 = h1 @ A2.T
    g3 = np.abs(np.asarray(dout, dtype=np.float64))
    g2 = g3 @ A3
    g1 = g2 @ A2
    return g1 @ A1, g1.T @ y, g2.T @ h1, g3.T @ h2
