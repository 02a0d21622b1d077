"""hashgrid_loss_grad (paper Section 4, "Training": squared error; mean absolute percentage error
|p - t| / (|t| + 0.01)) through the C ABI against oracle/loss_oracle.py.

Bars.  The kernel computes in fp32, the oracle in fp64, on the same fp32 inputs.  The sign of p - t is
exact in both, so the sign of every slope must agree and a perfect prediction gives exactly 0.  Squared
error: p - t is rounded once, doubled exactly and multiplied by the factor (one more rounding):
2^-23 of the slope's magnitude.  Percentage error: |t| + 0.01 (the constant itself rounded to fp32), a
division and a product: 4 roundings, 3e-7.  The sum of the loss values is taken in fp64 over fp32 values
of which each carries up to 4 roundings: 3e-7 of the sum.
"""

import numpy as np
import pytest
import torch

from oracle import loss_oracle as lo
from paper_2201_05989_amd import binding, loss_grad

pytestmark = pytest.mark.gpu

KINDS = {"l2": lo.L2, "mape": lo.MAPE}


def make(n, seed):
    rng = np.random.default_rng(seed)
    t = rng.normal(size=n).astype(np.float32)
    p = (t + rng.normal(size=n) * np.exp(rng.uniform(-12, 1, n))).astype(np.float32)
    p[::7] = t[::7]  # perfect predictions
    t[3::11] = 0.0  # targets on the surface: the offset alone is the denominator
    return p, t


@pytest.mark.parametrize("loss", ["l2", "mape"])
@pytest.mark.parametrize("n,shift", [(1, 0), (3, 0), (257, 0), (70001, 0), (70001, 1), (3 << 18, 0), (4096, 3)])
def test_slopes_and_loss_sum_against_the_oracle(loss, n, shift):
    p, t = make(n + shift, n)
    scale = 128.0 / n
    # shift > 0: views that start 4 * shift bytes into an allocation, so the kernel takes its scalar path
    pd, td = (torch.from_numpy(a).cuda()[shift:] for a in (p, t))
    out = torch.full((n + shift,), float("nan"), device="cuda")[shift:]
    total = torch.full((1,), 5.0, dtype=torch.float64, device="cuda")
    loss_grad(pd, td, loss, scale, out, total)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = lo.loss_grad(p[shift:], t[shift:], KINDS[loss], scale)
    assert np.array_equal(np.sign(got), np.sign(ref))
    assert (got[p[shift:] == t[shift:]] == 0).all()
    assert (np.abs(got - ref) <= 3e-7 * np.abs(ref)).all()
    ref_sum = lo.loss_values(p[shift:], t[shift:], KINDS[loss]).sum()
    assert abs(float(total.cpu()[0]) - 5.0 - ref_sum) <= 3e-7 * ref_sum + 1e-12
    # without the sum: the same slopes
    out2 = torch.empty_like(out)
    loss_grad(pd, td, KINDS[loss], scale, out2)
    assert torch.equal(out, out2)


def test_non_finite_values_propagate_and_bad_arguments_are_refused():
    p = torch.tensor([1.0, float("nan"), float("inf"), 2.0], device="cuda")
    t = torch.tensor([0.5, 0.0, 0.0, float("nan")], device="cuda")
    for loss in ("l2", "mape"):
        out = torch.zeros(4, device="cuda")
        loss_grad(p, t, loss, 1.0, out)
        got = out.cpu().numpy()
        assert np.isfinite(got[0]) and np.isnan(got[1]) and np.isnan(got[3])
        assert got[2] == (np.inf if loss == "l2" else 100.0)  # the percentage error's slope is bounded by 1 / offset
    lib = binding.load_library()
    out = torch.zeros(4, device="cuda")
    args = (p.data_ptr(), t.data_ptr())
    assert lib.hashgrid_loss_grad(4, *args, 2, 1.0, out.data_ptr(), None, None) == 1
    assert lib.hashgrid_loss_grad(4, *args, 0, float("inf"), out.data_ptr(), None, None) == 1
    assert lib.hashgrid_loss_grad(4, *args, 0, float("nan"), out.data_ptr(), None, None) == 1
    assert lib.hashgrid_loss_grad(4, p.data_ptr() + 2, t.data_ptr(), 0, 1.0, out.data_ptr(), None, None) == 1
    assert lib.hashgrid_loss_grad(4, *args, 0, 1.0, None, None, None) == 1
    eight = torch.zeros(2, dtype=torch.float64, device="cuda")
    assert lib.hashgrid_loss_grad(4, *args, 0, 1.0, out.data_ptr(), eight.data_ptr() + 4, None) == 1
    assert lib.hashgrid_loss_grad(0, None, None, 1, 1.0, None, None, None) == 0
    torch.cuda.synchronize()
    assert (out == 0).all()
