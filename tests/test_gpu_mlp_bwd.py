"""hashgrid_mlp_bwd (backward pass of the paper's 64-64 ReLU network, Section 4 "Architecture", on the
matrix cores) and hashgrid_encode_mlp_fwd_train, through the C ABI, against oracle/mlp_oracle.py.

Bars.  Where nothing rounds (small integers, multiples of 1/8: every half-precision operand is exact
and every fp32 sum is an integer or dyadic) the results must be equal.  Otherwise the kernel and the
oracle round the same values to half precision at the same points but accumulate in fp32 and fp64, so
a value next to a rounding boundary may land on the other side: every result is held to 2^-10 of the
sum of the absolute values along its chain (oracle bwd_magnitudes), and the median error to 1e-5 of
it.  Points with a hidden pre-activation next to zero are left out of the random cases: there the
ReLU mask itself, a discontinuity, could differ between fp32 and fp64 sums.
"""
import numpy as np
import pytest
import torch

from oracle import hashgrid_oracle as orc
from oracle import mlp_oracle as mlp
from paper_2201_05989_amd import HashGrid, mlp_bwd, synth

pytestmark = pytest.mark.gpu


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def run_gpu(y, W1, W2, W3, dout):
    B, n_in = y.shape
    n_out = W3.shape[0]
    dy = torch.full((B, n_in), float("nan"), dtype=torch.float16, device="cuda")
    dW1 = torch.zeros((64, n_in), device="cuda")
    dW2 = torch.zeros((64, 64), device="cuda")
    dW3 = torch.zeros((n_out, 64), device="cuda")
    mlp_bwd(dev(y, np.float16), dev(W1, np.float16), dev(W2, np.float16), dev(W3, np.float16), dev(dout, np.float32),
            dy, dW1, dW2, dW3)
    torch.cuda.synchronize()
    return [t.cpu().numpy().astype(np.float64) for t in (dy, dW1, dW2, dW3)]


@pytest.mark.parametrize("n_in,n_out,B", [(32, 1, 64), (32, 3, 1000), (8, 8, 33), (64, 32, 257), (40, 9, 4097), (16, 2, 31),
                                          (32, 17, 40000), (24, 1, 70001)])
def test_equal_to_the_oracle_where_nothing_rounds(n_in, n_out, B):
    # sparse small-integer weights, inputs and upstream gradients in multiples of 1/8 and 1/4: a permuted
    # operand, a transposed weight or a wrong ReLU mask changes the integers
    rng = np.random.default_rng(n_in * 100 + n_out)
    W1 = rng.integers(-1, 2, (64, n_in)) * (rng.random((64, n_in)) < 0.2)
    W2 = rng.integers(-1, 2, (64, 64)) * (rng.random((64, 64)) < 0.1)
    W3 = rng.integers(-2, 3, (n_out, 64))
    y = rng.integers(-8, 9, (B, n_in)) / 8.0
    dout = rng.integers(-4, 5, (B, n_out)) / 4.0
    ref = mlp.mlp_bwd(y, W1, W2, W3, dout)
    assert all(np.abs(r).max() > 0 for r in ref)
    got = run_gpu(y, W1, W2, W3, dout)
    # fp32 sums of dyadic numbers of this size are exact; gradients are multiples of 1/4: exact in fp16 below 512
    assert np.abs(ref[0]).max() < 512
    for g, r in zip(got, ref):
        np.testing.assert_array_equal(g, r)
    # calling again accumulates the weight gradients and rewrites dL/dy
    Bt = torch.cuda
    dy = torch.zeros((B, n_in), dtype=torch.float16, device="cuda")
    dWs = [dev(a, np.float32) for a in got[1:]]
    mlp_bwd(dev(y, np.float16), dev(W1, np.float16), dev(W2, np.float16), dev(W3, np.float16), dev(dout, np.float32),
            dy, *dWs)
    Bt.synchronize()
    np.testing.assert_array_equal(dy.cpu().numpy().astype(np.float64), ref[0])
    for t, r in zip(dWs, ref[1:]):
        np.testing.assert_array_equal(t.cpu().numpy().astype(np.float64), 2 * r)


def test_every_served_shape_and_weights_at_any_alignment():
    # every n_in (multiples of 8 up to 64) with a spread of n_out, exact as above; the weight matrices start
    # 2 bytes into their allocations (the staging then reads them half by half instead of in 8-byte pieces)
    rng = np.random.default_rng(5)
    for n_in in range(8, 65, 8):
        for n_out in (1, 7, 8, 9, 16, 25, 32):
            B = int(rng.integers(1, 400))
            W1 = rng.integers(-1, 2, (64, n_in)) * (rng.random((64, n_in)) < 0.2)
            W2 = rng.integers(-1, 2, (64, 64)) * (rng.random((64, 64)) < 0.1)
            W3 = rng.integers(-2, 3, (n_out, 64))
            y = rng.integers(-8, 9, (B, n_in)) / 8.0
            dout = rng.integers(-4, 5, (B, n_out)) / 4.0
            ref = mlp.mlp_bwd(y, W1, W2, W3, dout)

            def shifted(a):
                buf = torch.zeros(a.size + 1, dtype=torch.float16, device="cuda")
                buf[1:] = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float16).ravel()).cuda()
                return buf[1:].view(*a.shape)

            dy = torch.full((B, n_in), float("nan"), dtype=torch.float16, device="cuda")
            dWs = [torch.zeros((64, n_in), device="cuda"), torch.zeros((64, 64), device="cuda"),
                   torch.zeros((n_out, 64), device="cuda")]
            Ws = [shifted(W1), shifted(W2), shifted(W3)]
            assert all(w_.data_ptr() % 4 == 2 for w_ in Ws)
            mlp_bwd(dev(y, np.float16), *Ws, dev(dout, np.float32), dy, *dWs)
            torch.cuda.synchronize()
            for g, r in zip([dy] + dWs, ref):
                np.testing.assert_array_equal(g.cpu().numpy().astype(np.float64), r, err_msg=f"n_in={n_in} n_out={n_out} B={B}")


@pytest.mark.parametrize("n_in,n_out,B", [(32, 1, 20000), (32, 4, 5000), (64, 16, 3000), (24, 3, 777)])
def test_random_networks_within_the_rounding_bound(n_in, n_out, B):
    rng = np.random.default_rng(7 * n_in + n_out)
    W1 = (rng.standard_normal((64, n_in)) * np.sqrt(2.0 / n_in)).astype(np.float16)
    W2 = (rng.standard_normal((64, 64)) * np.sqrt(2.0 / 64)).astype(np.float16)
    W3 = (rng.standard_normal((n_out, 64)) / 8.0).astype(np.float16)
    y = rng.uniform(-1, 1, (B, n_in)).astype(np.float16)
    dout = rng.standard_normal((B, n_out)).astype(np.float32)
    # leave out points with a pre-activation next to the ReLU kink (see the module's header)
    y64, A1, A2 = y.astype(np.float64), W1.astype(np.float64), W2.astype(np.float64)
    a1 = y64 @ A1.T
    h1 = np.maximum(a1, 0).astype(np.float16).astype(np.float64)
    a2 = h1 @ A2.T
    keep = (np.abs(a1).min(axis=1) > 1e-4) & (np.abs(a2).min(axis=1) > 1e-4)
    assert keep.mean() > 0.9
    y, dout = y[keep], dout[keep]
    ref = mlp.mlp_bwd(y, W1, W2, W3, dout)
    mags = mlp.bwd_magnitudes(y, W1, W2, W3, dout)
    got = run_gpu(y, W1, W2, W3, dout)
    for name, g, r, m in zip(("dy", "dW1", "dW2", "dW3"), got, ref, mags):
        err = np.abs(g - r)
        bound = 2.0 ** -10 * m + (2.0 ** -11 * np.abs(r) + 2.0 ** -24 if name == "dy" else 0.0)
        assert (err <= bound + 1e-30).all(), f"{name}: {int((err > bound).sum())} of {err.size} off, worst {np.max(err / (m + 1e-300)):.2e}"
        assert np.median(err / (m + 1e-300)) <= (3e-4 if name == "dy" else 1e-5), name  # dy: its own fp16 rounding


def test_training_forward_keeps_the_encoded_features_and_feeds_the_backward_passes():
    # encode_mlp_fwd_train: out as encode_mlp_fwd, y as encode_fwd; then mlp_bwd and encode_bwd: the table
    # gradient of the whole model against the oracles chained the same way
    w = synth.WORKLOADS["sdf3d"]
    B = 5000
    cfg = orc.OracleConfig(w.d, w.L, w.F, w.T, w.N_min, w.N_max)
    grid = HashGrid(w.d, w.L, w.F, w.T, w.N_min, w.N_max, "f16", "f16")
    x, theta, _ = synth.make_inputs(w, grid.n_entries, B=B, table_scale=1.0)
    rng = np.random.default_rng(3)
    n_in, n_out = w.L * w.F, 2
    W1 = (rng.standard_normal((64, n_in)) * np.sqrt(2.0 / n_in)).astype(np.float16)
    W2 = (rng.standard_normal((64, 64)) * np.sqrt(2.0 / 64)).astype(np.float16)
    W3 = (rng.standard_normal((n_out, 64)) / 8.0).astype(np.float16)
    xd, td = dev(x, np.float32), dev(theta, np.float16)
    Wd = [dev(a, np.float16) for a in (W1, W2, W3)]
    out_plain = grid.encode_mlp_fwd(xd, td, *Wd)
    yk = torch.empty((B, n_in), dtype=torch.float16, device="cuda")
    out = grid.encode_mlp_fwd(xd, td, *Wd, y=yk)
    assert torch.equal(out, out_plain)
    y_enc = grid.encode_fwd(xd, td)
    ne = yk != y_enc  # two kernels, the same fp32 arithmetic: at most a last-bit difference on exact ties
    assert int(ne.sum()) <= max(8, yk.numel() // 10000)
    # backward: dL/dout = out (loss = |out|^2 / 2)
    dy = torch.empty_like(yk)
    dWs = [torch.zeros((64, n_in), device="cuda"), torch.zeros((64, 64), device="cuda"), torch.zeros((n_out, 64), device="cuda")]
    mlp_bwd(yk, *Wd, out, dy, *dWs)
    g = grid.encode_bwd(xd, dy, use_workspace=True)
    torch.cuda.synchronize()
    y_np, out_np, dy_np = yk.cpu().numpy(), out.cpu().numpy(), dy.cpu().numpy()
    # each stage against its oracle, fed with the GPU's own inputs to that stage
    ref = mlp.mlp_bwd(y_np, W1, W2, W3, out_np)
    mags = mlp.bwd_magnitudes(y_np, W1, W2, W3, out_np)
    bad = np.abs(dy_np.astype(np.float64) - ref[0]) > 2.0 ** -10 * mags[0] + 2.0 ** -11 * np.abs(ref[0]) + 2.0 ** -24
    assert bad.mean() < 1e-3  # (points next to a ReLU kink are not filtered here)
    g_ref = orc.encode_bwd(cfg, x, dy_np)
    g_abs = orc.encode_bwd(cfg, x, np.abs(dy_np.astype(np.float64)))
    H = max(3 + int(np.ceil(np.log2(B))), 11)
    floor = float(np.abs(dy_np.astype(np.float64)).max()) * 2.0 ** (H - 54)
    assert (np.abs(g.cpu().numpy().astype(np.float64) - g_ref) <= 1e-5 * g_abs + floor + 1e-30).all()


def test_argument_checks():
    from paper_2201_05989_amd import binding
    lib = binding.load_library()
    p = 4096
    assert lib.hashgrid_mlp_bwd(0, 32, 1, None, None, None, None, None, None, None, None, None, None) == 0
    assert lib.hashgrid_mlp_bwd(8, 32, 1, None, p, p, p, p, p, p, p, p, None) == 1
    assert lib.hashgrid_mlp_bwd(8, 12, 1, p, p, p, p, p, p, p, p, p, None) == 2   # n_in not a multiple of 8
    assert lib.hashgrid_mlp_bwd(8, 72, 1, p, p, p, p, p, p, p, p, p, None) == 2
    assert lib.hashgrid_mlp_bwd(8, 32, 33, p, p, p, p, p, p, p, p, p, None) == 2
    assert lib.hashgrid_mlp_bwd(8, 32, 0, p, p, p, p, p, p, p, p, p, None) == 1
    assert lib.hashgrid_mlp_bwd(8, 32, 1, p + 8, p, p, p, p, p, p, p, p, None) == 1  # y not 16-byte aligned
