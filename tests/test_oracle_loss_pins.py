"""Pins of the loss oracle (paper Section 4, "Training": squared error; mean absolute percentage error
|p - t| / (|t| + 0.01)) against things other than itself: hand-computed values, central differences of
the loss values, a library's autograd, and the properties the definitions imply."""
import numpy as np
import pytest
import torch

from oracle import loss_oracle as lo


def test_hand_computed_values():
    # squared error: (3 - 1)^2 = 4, slope 2 * 2 = 4; (−0.5 − 0.25)^2 = 0.5625, slope −1.5
    assert lo.loss_values([3.0, -0.5], [1.0, 0.25], lo.L2).tolist() == [4.0, 0.5625]
    assert lo.loss_grad([3.0, -0.5], [1.0, 0.25], lo.L2).tolist() == [4.0, -1.5]
    # percentage error: |0.5 − 0.99| / (0.99 + 0.01) = 0.49, slope −1; target −0.19: |0 + 0.19| / 0.2 = 0.95, slope +5;
    # target 0: the offset alone is the denominator, |0.001| / 0.01 = 0.1, slope 100
    v = lo.loss_values([0.5, 0.0, 0.001], [0.99, -0.19, 0.0], lo.MAPE)
    g = lo.loss_grad([0.5, 0.0, 0.001], [0.99, -0.19, 0.0], lo.MAPE)
    assert np.allclose(v, [0.49, 0.95, 0.1], rtol=1e-15, atol=0)
    assert np.allclose(g, [-1.0, 5.0, 100.0], rtol=1e-15, atol=0)


@pytest.mark.parametrize("kind", [lo.L2, lo.MAPE])
def test_gradient_is_the_central_difference_of_the_values(kind):
    rng = np.random.default_rng(5)
    p, t = rng.normal(size=2000), rng.normal(size=2000)
    h = 1e-6
    keep = np.abs(p - t) > 10 * h  # the percentage error has a kink at p = t
    num = (lo.loss_values(p + h, t, kind) - lo.loss_values(p - h, t, kind)) / (2 * h)
    g = lo.loss_grad(p, t, kind)
    assert np.allclose(g[keep], num[keep], rtol=1e-8, atol=1e-8)
    assert np.array_equal(lo.loss_grad(p, t, kind, scale=0.125), 0.125 * g)  # the factor multiplies, exactly for a power of two


def test_a_library_agrees():
    rng = np.random.default_rng(6)
    p = torch.tensor(rng.normal(size=(64, 3)), dtype=torch.float64, requires_grad=True)
    t = torch.tensor(rng.normal(size=(64, 3)), dtype=torch.float64)
    torch.nn.functional.mse_loss(p, t, reduction="sum").backward()
    assert np.allclose(lo.loss_grad(p.detach().numpy(), t.numpy(), lo.L2), p.grad.numpy(), rtol=1e-15, atol=0)
    assert np.isclose(lo.loss_values(p.detach().numpy(), t.numpy(), lo.L2).sum(),
                      float(torch.nn.functional.mse_loss(p.detach(), t, reduction="sum")), rtol=1e-14)
    p.grad = None
    ((p - t).abs() / (t.abs() + 0.01)).sum().backward()
    assert np.allclose(lo.loss_grad(p.detach().numpy(), t.numpy(), lo.MAPE), p.grad.numpy(), rtol=1e-15, atol=0)


def test_properties_of_the_definitions():
    rng = np.random.default_rng(7)
    p, t = rng.normal(size=500), rng.normal(size=500)
    for kind in (lo.L2, lo.MAPE):
        assert (lo.loss_values(p, t, kind) >= 0).all()
        assert (lo.loss_values(t, t, kind) == 0).all() and (lo.loss_grad(t, t, kind) == 0).all()  # a perfect prediction stays
        # a step against the gradient lowers the loss
        g = lo.loss_grad(p, t, kind)
        assert (lo.loss_values(p - 1e-4 * np.sign(g), t, kind) <= lo.loss_values(p, t, kind)).all()
    # squared error is symmetric in its arguments, the percentage error is not: it is relative to the target
    assert np.array_equal(lo.loss_values(p, t, lo.L2), lo.loss_values(t, p, lo.L2))
    assert np.allclose(lo.loss_values(10 * p, 10 * t, lo.MAPE) * (np.abs(10 * t) + 0.01),
                       10 * lo.loss_values(p, t, lo.MAPE) * (np.abs(t) + 0.01), rtol=1e-13)
    # far from zero the percentage error is scale-free: scaling both by 1000 changes it by the offset's share only
    big = np.abs(t) > 0.5
    r = lo.loss_values(1000 * p[big], 1000 * t[big], lo.MAPE) / lo.loss_values(p[big], t[big], lo.MAPE)
    assert np.all((r > 1.0) & (r < 1.021))
    with pytest.raises(ValueError):
        lo.loss_values(p, t, 2)
