"""CPU oracle of the training losses (paper Section 4, "Training"): the squared error used for images
and radiance fields, and the mean absolute percentage error used for signed distance functions,
|prediction - target| / (|target| + 0.01).  TEST INFRASTRUCTURE ONLY: the test-suite uses it; the GPU
library never does.

Arithmetic: the definitions written out in numpy fp64, one scalar of the network's output at a time;
the derivative is the textbook one (2 (p - t); sign(p - t) / (|t| + 0.01), with sign(0) = 0, the
subgradient that leaves a perfect prediction alone).  The paper takes means over the batch; here, as
at the library's boundary, the caller chooses the factor (`scale`, e.g. 1/n, times any loss scaling
of half-precision training) and the loss values are returned per scalar so that a test can sum them
as it likes.  The luminance-relative loss of neural radiance caching is defined in another paper and
is not part of this oracle.
"""
from __future__ import annotations

import numpy as np

L2, MAPE = 0, 1
MAPE_OFFSET = 0.01  # Section 4, "Training": the constant in the denominator of the percentage error


def loss_values(prediction, target, kind: int) -> np.ndarray:
    """Per-scalar loss, fp64, same shape as the inputs."""
    p = np.asarray(prediction, dtype=np.float64)
    t = np.asarray(target, dtype=np.float64)
    if kind == L2:
        return (p - t) ** 2
    if kind == MAPE:
        return np.abs(p - t) / (np.abs(t) + MAPE_OFFSET)
    raise ValueError("unknown loss")


def loss_grad(prediction, target, kind: int, scale: float = 1.0) -> np.ndarray:
    """scale * d loss / d prediction per scalar, fp64."""
    p = np.asarray(prediction, dtype=np.float64)
    t = np.asarray(target, dtype=np.float64)
    if kind == L2:
        return scale * 2.0 * (p - t)
    if kind == MAPE:
        return scale * np.sign(p - t) / (np.abs(t) + MAPE_OFFSET)
    raise ValueError("unknown loss")
