"""Parity of hashgrid_adam_step (fp32 on the GPU) with the fp64 oracle, scalar by scalar.

Bars: second moment within 2e-6 relative, first moment within 2e-6 of the magnitude of its two
summands (beta1 |m| + (1 - beta1) |g|: they may cancel), +1e-37 near the fp32 subnormal range;
master value within 4e-6 * lr (the step is at most a few lr; its fp32 evaluation has a few
ulps of relative error) + 1e-7 |theta*|; the half copy equals the GPU's own master value
rounded to nearest even, bit for bit; skipped scalars keep every bit."""
import numpy as np
import pytest
import torch

from oracle import hashgrid_oracle as orc
from paper_2201_05989_amd import adam_step, binding

pytestmark = pytest.mark.gpu


def run(n, steps, lr, zero_frac, seed, zero_grad=True, with_half=True):
    rng = np.random.default_rng(seed)
    theta = rng.uniform(-1e-4, 1e-4, n).astype(np.float32)   # the paper's initialisation
    p = torch.from_numpy(theta.copy()).cuda()
    ph = p.half() if with_half else None
    m = torch.zeros(n, device="cuda")
    v = torch.zeros(n, device="cuda")
    t64, m64, v64 = theta.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, steps + 1):
        g = (rng.standard_normal(n) * 10.0 ** rng.uniform(-7, 1, n)).astype(np.float32)
        g[rng.random(n) < zero_frac] = 0.0
        gd = torch.from_numpy(g.copy()).cuda()
        before = (p.clone(), m.clone(), v.clone(), None if ph is None else ph.clone())
        adam_step(p, gd, m, v, step, lr=lr, params_half=ph, zero_grad=zero_grad)
        m_scale = 0.9 * np.abs(m64) + 0.1 * np.abs(g.astype(np.float64))
        orc.adam_step(t64, g, m64, v64, lr=lr, step=step)
        torch.cuda.synchronize()
        skipped = torch.from_numpy(g == 0).cuda()
        assert torch.equal(p[skipped], before[0][skipped]) and torch.equal(m[skipped], before[1][skipped])
        assert torch.equal(v[skipped], before[2][skipped])
        if ph is not None:
            assert torch.equal(ph[skipped], before[3][skipped])
            assert torch.equal(ph[~skipped], p[~skipped].half())
        assert bool((gd == 0).all()) if zero_grad else torch.equal(gd.cpu(), torch.from_numpy(g))
        pm, pv, pp = m.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64), p.cpu().numpy().astype(np.float64)
        assert (np.abs(pm - m64) <= 2e-6 * m_scale + 1e-37).all()
        assert (np.abs(pv - v64) <= 2e-6 * np.abs(v64) + 1e-37).all()
        assert (np.abs(pp - t64) <= 4e-6 * lr * step + 1e-7 * np.abs(t64)).all()
        # keep both sides on the same trajectory: continue from the GPU's state (exactly representable in fp64)
        t64, m64, v64 = pp.copy(), pm.copy(), pv.copy()


@pytest.mark.parametrize("n,zero_frac", [(1, 0.0), (3, 0.0), (4, 0.0), (1027, 0.3), (100003, 0.9), (1 << 20, 0.1)])
def test_adam_matches_oracle(n, zero_frac):
    run(n, steps=4, lr=1e-2, zero_frac=zero_frac, seed=n)


def test_adam_sdf_learning_rate_no_half_copy_keep_grad():
    run(50000, steps=3, lr=1e-4, zero_frac=0.5, seed=5, zero_grad=False, with_half=False)


def test_adam_full_table_size_of_the_headline_configuration():
    run(6098925 * 2, steps=2, lr=1e-2, zero_frac=0.02, seed=9)


def test_adam_argument_checks():
    lib = binding.load_library()
    cfg = binding.hashgrid_adam_config(1e-2, 0.9, 0.99, 1e-15, 0.0)
    import ctypes
    a = torch.zeros(64, device="cuda")
    ptr = a.data_ptr()
    ok = lambda *args: lib.hashgrid_adam_step(*args)
    assert ok(0, None, None, None, None, None, ctypes.byref(cfg), 1, 1, None) == 0
    assert ok(64, ptr, None, ptr, ptr, ptr, ctypes.byref(cfg), 0, 1, None) == 1      # step 0
    assert ok(64, None, None, ptr, ptr, ptr, ctypes.byref(cfg), 1, 1, None) == 1     # NULL master
    assert ok(60, ptr + 4, None, ptr, ptr, ptr, ctypes.byref(cfg), 1, 1, None) == 1  # misaligned
    bad = binding.hashgrid_adam_config(1e-2, 1.0, 0.99, 1e-15, 0.0)
    assert ok(64, ptr, None, ptr, ptr, ptr, ctypes.byref(bad), 1, 1, None) == 1      # beta1 = 1


@pytest.mark.parametrize("n,scale", [(5, 1.0), (100003, 1.0 / 128.0), (1 << 18, 1.0 / 1024.0)])
def test_adam_on_half_precision_gradients(n, scale):
    # the gradient as the backward passes write it with grad_dtype fp16, scaled by the caller's loss scale: the
    # step uses float(g16) * scale (exact for a power of two); the oracle gets exactly those values
    rng = np.random.default_rng(n)
    theta = rng.uniform(-1e-4, 1e-4, n).astype(np.float32)
    p = torch.from_numpy(theta.copy()).cuda()
    ph, m, v = p.half(), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    t64, m64, v64 = theta.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, 4):
        g16 = np.clip((rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 2, n)) / scale, -6e4, 6e4).astype(np.float16)
        g16[rng.random(n) < 0.3] = 0.0
        g16[~np.isfinite(g16)] = 0.0
        g = g16.astype(np.float64) * scale
        gd = torch.from_numpy(g16.copy()).cuda()
        before = (p.clone(), m.clone(), v.clone(), ph.clone())
        zero = step != 2
        adam_step(p, gd, m, v, step, lr=1e-2, params_half=ph, zero_grad=zero, grad_scale=scale)
        m_scale = 0.9 * np.abs(m64) + 0.1 * np.abs(g)
        orc.adam_step(t64, g, m64, v64, lr=1e-2, step=step)
        torch.cuda.synchronize()
        skipped = torch.from_numpy(g16 == 0).cuda()
        for now, was in zip((p, m, v, ph), before):
            assert torch.equal(now[skipped], was[skipped])
        assert torch.equal(ph[~skipped], p[~skipped].half())
        assert bool((gd == 0).all()) if zero else torch.equal(gd.cpu(), torch.from_numpy(g16))
        pm, pv, pp = (a.cpu().numpy().astype(np.float64) for a in (m, v, p))
        assert (np.abs(pm - m64) <= 2e-6 * m_scale + 1e-37).all()
        assert (np.abs(pv - v64) <= 2e-6 * np.abs(v64) + 1e-37).all()
        assert (np.abs(pp - t64) <= 4e-6 * 1e-2 * step + 1e-7 * np.abs(t64)).all()
        t64, m64, v64 = pp.copy(), pm.copy(), pv.copy()
    lib = binding.load_library()
    cfg = binding.hashgrid_adam_config(1e-2, 0.9, 0.99, 1e-15, 0.0)
    import ctypes
    a = p.data_ptr()
    assert lib.hashgrid_adam_step_half_grad(4, a, None, a, a, a, ctypes.byref(cfg), 1, 1, 0.0, None) == 1    # scale 0
    assert lib.hashgrid_adam_step_half_grad(4, a, None, a + 2, a, a, ctypes.byref(cfg), 1, 1, 1.0, None) == 1  # misaligned
    assert lib.hashgrid_adam_step_half_grad(0, None, None, None, None, None, ctypes.byref(cfg), 1, 1, 1.0, None) == 0


@pytest.mark.parametrize("l2", [1e-6, 1e-2])
def test_adam_with_the_l2_regularisation_of_the_network_weights(l2):
    # Section 4, "Training": factor 1e-6 on the network's weights; here on 6208 scalars (the 64-64 network with 32
    # inputs and one output), some gradients exactly zero: those weights still move, by the regulariser alone
    rng = np.random.default_rng(11)
    n = 64 * 32 + 64 * 64 + 64
    theta = (rng.standard_normal(n) * 0.2).astype(np.float32)
    p = torch.from_numpy(theta.copy()).cuda()
    ph, m, v = p.half(), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    t64, m64, v64 = theta.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, 5):
        g = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 0, n)).astype(np.float32)
        g[rng.random(n) < 0.2] = 0.0
        gd = torch.from_numpy(g.copy()).cuda()
        before = p.clone()
        adam_step(p, gd, m, v, step, lr=1e-3, params_half=ph, l2_reg=l2)
        # the gradient with the regulariser's term is a sum that may cancel: errors are measured against its summands
        g_mass = np.abs(g.astype(np.float64)) + l2 * np.abs(t64)
        m_scale = 0.9 * np.abs(m64) + 0.1 * g_mass
        v_scale = 0.99 * v64 + 0.01 * g_mass ** 2
        orc.adam_step(t64, g, m64, v64, lr=1e-3, step=step, l2=l2)
        torch.cuda.synchronize()
        assert bool((gd == 0).all()) and torch.equal(ph, p.half())
        moved = (p != before).cpu().numpy()
        assert moved[(g == 0) & (np.abs(theta) > 1e-3)].all()   # (theta far from 0: l2 * theta is not lost in eps)
        pm, pv, pp = (a.cpu().numpy().astype(np.float64) for a in (m, v, p))
        assert (np.abs(pm - m64) <= 4e-6 * m_scale + 1e-37).all()
        assert (np.abs(pv - v64) <= 4e-6 * v_scale + 1e-37).all()
        # the step is lr * m_hat / sqrt(v_hat): where the two terms of the gradient nearly cancel its relative error is
        # that of the small difference; everywhere it is at most a few lr
        well = np.abs(g.astype(np.float64) + l2 * t64) > 1e-3 * g_mass
        assert (np.abs(pp - t64)[well] <= 4e-5 * 1e-3 * step + 1e-7 * np.abs(t64[well])).all()
        assert (np.abs(pp - t64) <= 1e-2 * 1e-3 * step + 1e-7 * np.abs(t64)).all()
        t64, m64, v64 = pp.copy(), pm.copy(), pv.copy()
    lib = binding.load_library()
    import ctypes
    bad = binding.hashgrid_adam_config(1e-2, 0.9, 0.99, 1e-15, -1.0)
    a = p.data_ptr()
    assert lib.hashgrid_adam_step(4, a, None, a, a, a, ctypes.byref(bad), 1, 1, None) == 1
