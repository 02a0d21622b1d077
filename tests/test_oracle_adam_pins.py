"""Pins for the oracle's optimiser step (paper Section 4, "Training": Adam with
beta1 = 0.9, beta2 = 0.99, eps = 1e-15, entries with an exactly-zero gradient
skipped).  Closed forms of Adam's recurrences, the skip rule, and an independent
library implementation (torch.optim.Adam on the CPU, fp64) as a third opinion."""
import numpy as np
import torch

from oracle import hashgrid_oracle as orc

B1, B2, EPS = 0.9, 0.99, 1e-15


def test_first_step_is_lr_times_sign():
    # t = 1 from zero moments: m_hat = g, v_hat = g^2, so the update is lr * g / (|g| + eps)
    g = np.array([3.0, -0.25, 1e-6, -1e-12, 1e-15])
    theta = np.zeros(5)
    m, v = np.zeros(5), np.zeros(5)
    orc.adam_step(theta, g, m, v, lr=1e-2, step=1)
    np.testing.assert_allclose(theta, -1e-2 * g / (np.abs(g) + EPS), rtol=1e-14)
    # eps = 1e-15 only matters for gradients of that size: |g| = eps gives exactly half a step
    np.testing.assert_allclose(theta[4], -0.5e-2, rtol=1e-12)
    np.testing.assert_allclose(m, (1 - B1) * g, rtol=1e-15)
    np.testing.assert_allclose(v, (1 - B2) * g * g, rtol=1e-15)


def test_constant_gradient_closed_form():
    # constant g: m_t = g (1 - b1^t), v_t = g^2 (1 - b2^t): the corrected ratio is sign(g) at every step
    g = np.array([0.7, -2.0])
    theta = np.array([1.0, 1.0])
    m, v = np.zeros(2), np.zeros(2)
    for t in range(1, 51):
        orc.adam_step(theta, g, m, v, lr=1e-3, step=t)
        np.testing.assert_allclose(m, g * (1 - B1 ** t), rtol=1e-13)
        np.testing.assert_allclose(v, g * g * (1 - B2 ** t), rtol=1e-13)
    np.testing.assert_allclose(theta, 1.0 - 50 * 1e-3 * np.sign(g), rtol=1e-12)


def test_zero_gradient_entries_are_skipped_bit_for_bit():
    rng = np.random.default_rng(0)
    theta = rng.standard_normal(1000)
    m = rng.standard_normal(1000)      # non-zero moments: plain Adam would still move these entries
    v = rng.random(1000)
    g = rng.standard_normal(1000)
    g[::3] = 0.0
    t0, m0, v0 = theta.copy(), m.copy(), v.copy()
    orc.adam_step(theta, g, m, v, lr=1e-2, step=7)
    skipped = g == 0
    assert (theta[skipped] == t0[skipped]).all() and (m[skipped] == m0[skipped]).all() and (v[skipped] == v0[skipped]).all()
    assert (theta[~skipped] != t0[~skipped]).all()


def test_matches_library_adam_when_no_gradient_is_zero():
    rng = np.random.default_rng(1)
    n = 5000
    theta0 = rng.uniform(-1e-4, 1e-4, n)
    theta = theta0.copy()
    m, v = np.zeros(n), np.zeros(n)
    p = torch.tensor(theta0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=1e-2, betas=(B1, B2), eps=EPS, weight_decay=0.0)
    for t in range(1, 21):
        g = rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 0, n)
        orc.adam_step(theta, g, m, v, lr=1e-2, step=t)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-10, atol=1e-14)


def test_rejects_step_zero():
    a = np.zeros(3)
    try:
        orc.adam_step(a, a.copy(), a.copy(), a.copy(), lr=1e-2, step=0)
        assert False
    except ValueError:
        pass


def test_l2_regularisation_is_the_library_weight_decay_and_a_closed_form():
    # Section 4, "Training": L2 regularisation (factor 1e-6) on the network's weights.  As a term l2 * theta in
    # the gradient it is what torch.optim.Adam calls weight_decay (fp64 on the CPU as a third opinion) ...
    rng = np.random.default_rng(4)
    n = 3000
    theta0 = rng.standard_normal(n) * 0.3
    for l2 in (1e-6, 0.05):
        theta, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
        p = torch.tensor(theta0, dtype=torch.float64, requires_grad=True)
        opt = torch.optim.Adam([p], lr=1e-2, betas=(B1, B2), eps=EPS, weight_decay=l2)
        for t in range(1, 16):
            g = rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 0, n)
            orc.adam_step(theta, g, m, v, lr=1e-2, step=t, l2=l2)
            p.grad = torch.tensor(g, dtype=torch.float64)
            opt.step()
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-10, atol=1e-14)
    # ... and with no data gradient the first step moves every weight by lr towards zero (g' = l2 * theta, so the
    # update is lr * sign(theta) as long as |l2 * theta| >> eps), while l2 = 0 leaves it where it is
    theta = np.array([2.0, -0.5, 1e-3])
    m, v = np.zeros(3), np.zeros(3)
    orc.adam_step(theta, np.zeros(3), m, v, lr=1e-2, step=1, l2=1e-6)
    np.testing.assert_allclose(theta, np.array([2.0, -0.5, 1e-3]) - 1e-2 * np.sign([2.0, -0.5, 1e-3]), rtol=1e-5)
    np.testing.assert_allclose(m, 0.1 * 1e-6 * np.array([2.0, -0.5, 1e-3]), rtol=1e-12)
    theta = np.array([2.0, -0.5])
    m, v = np.zeros(2), np.zeros(2)
    orc.adam_step(theta, np.zeros(2), m, v, lr=1e-2, step=1)
    assert (theta == [2.0, -0.5]).all() and (m == 0).all()
