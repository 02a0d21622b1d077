"""The whole training step through the C ABI, many times in a row (paper Section 4: encoding + network forward,
loss, backward through network and encoding, Adam on tables and weights with the paper's hyper-parameters): the
model must learn.  Every call is held to the oracle by the parity tests; what only this test sees is that the calls
fit together (layouts, scales, the half-precision working copies following their master copies) over hundreds of
steps.  Targets are synthetic closed forms standing in for the paper's image and signed-distance data:

* a 2-D "image" with sharp edges and fine stripes, squared error (as for the gigapixel task), with one and with
  three output channels;
* the signed distance to a sphere in 3-D, mean absolute percentage error (as for the SDF task).

Bars are on the trend, with a wide margin under what a run reaches (the weight gradients are summed with
atomics, so runs differ in their last bits): the loss on fresh points falls by the stated factor, and the image
fit ends well below what the best constant prediction gives.
"""
import numpy as np
import pytest
import torch

from paper_2201_05989_amd import HashGrid, adam_step, loss_grad, mlp_bwd

pytestmark = pytest.mark.gpu


def image(x):
    # blocks of a 6 x 6 checkerboard, a disc, and fine diagonal stripes: edges that a smooth network alone blurs
    board = ((torch.floor(6 * x[:, 0]) + torch.floor(6 * x[:, 1])) % 2)
    disc = (((x[:, 0] - 0.5) ** 2 + (x[:, 1] - 0.45) ** 2) < 0.09).float()
    stripes = 0.25 * torch.sin(150.0 * (x[:, 0] + x[:, 1]))
    return (0.5 * board + 0.4 * disc + stripes).unsqueeze(1).contiguous()


def colour_image(x):
    # three channels that share edges but differ in phase and scale, as the channels of a photograph do
    g = image(x)[:, 0]
    return torch.stack([g, 0.8 * g + 0.1 * torch.sin(40.0 * x[:, 0]), 1.0 - g], dim=1).contiguous()


def sphere(x):
    return (torch.linalg.norm(x - 0.5, dim=1) - 0.3).unsqueeze(1).contiguous()


def train(d, L, T, N_max, target, loss, lr, steps, B, seed, n_out=1):
    torch.manual_seed(seed)
    F, n_in = 2, 2 * L
    grid = HashGrid(d, L, F, T, 16, N_max, "f16", "f16")
    tab = (torch.rand((grid.n_entries, F), device="cuda") * 2e-4 - 1e-4)  # Section 4, "Initialization"
    tab16, tab_g = tab.half(), torch.zeros_like(tab)
    tab_m, tab_v = torch.zeros_like(tab), torch.zeros_like(tab)
    shapes = [(64, n_in), (64, 64), (n_out, 64)]
    init = [(torch.rand(s, device="cuda") * 2 - 1) * np.sqrt(6.0 / (s[0] + s[1])) for s in shapes]  # Glorot and Bengio
    net = torch.cat([a.reshape(-1) for a in init]).contiguous()
    net16, net_g = net.half(), torch.zeros_like(net)
    net_m, net_v = torch.zeros_like(net), torch.zeros_like(net)

    def views(flat):
        out, at = [], 0
        for r, c in shapes:
            out.append(flat[at:at + r * c].view(r, c))
            at += r * c
        return out

    W, dW = views(net16), views(net_g)
    out = torch.empty((B, n_out), device="cuda")
    dout = torch.empty_like(out)
    y = torch.empty((B, n_in), dtype=torch.float16, device="cuda")
    dy = torch.empty_like(y)
    total = torch.zeros(1, dtype=torch.float64, device="cuda")
    history = []
    for step in range(1, steps + 1):
        x = torch.rand((B, d), device="cuda")
        t = target(x)
        grid.encode_mlp_fwd(x, tab16, *W, out, y=y)
        total.zero_()
        # the gradient of the summed loss: Adam does not care about the factor, and 1/B would push dL/dout, which
        # the network's backward pass rounds to half precision, into the subnormals
        loss_grad(out, t, loss, 1.0, dout, total)
        mlp_bwd(y, *W, dout, dy, *dW)
        grid.encode_bwd(x, dy, tab_g, overwrite=True)
        adam_step(tab, tab_g, tab_m, tab_v, step, lr=lr, params_half=tab16, zero_grad=False)
        adam_step(net, net_g, net_m, net_v, step, lr=lr, params_half=net16, zero_grad=True, l2_reg=1e-6)
        history.append(float(total.cpu()[0]) / (B * n_out))
    assert torch.isfinite(tab).all() and torch.isfinite(net).all()
    assert torch.equal(tab16, tab.half()) and torch.equal(net16, net.half())  # the working copies follow their masters
    return history


def test_an_image_is_learned_with_the_squared_error():
    h = train(d=2, L=16, T=1 << 17, N_max=1024, target=image, loss="l2", lr=1e-2, steps=400, B=1 << 14, seed=1)
    first, last = np.mean(h[:3]), np.mean(h[-10:])
    x = torch.rand((1 << 16, 2), device="cuda")
    variance = float(image(x).var())  # what the best constant prediction leaves
    print(f"image: loss {first:.4f} -> {last:.5f}; variance of the target {variance:.4f}")
    assert last < first / 30 and last < variance / 20


def test_three_output_channels_are_learned_together():
    h = train(d=2, L=16, T=1 << 17, N_max=1024, target=colour_image, loss="l2", lr=1e-2, steps=400, B=1 << 14, seed=3,
              n_out=3)
    first, last = np.mean(h[:3]), np.mean(h[-10:])
    print(f"colour image: loss {first:.4f} -> {last:.5f}")
    assert last < first / 30


def test_a_signed_distance_is_learned_with_the_percentage_error():
    h = train(d=3, L=16, T=1 << 15, N_max=256, target=sphere, loss="mape", lr=1e-3, steps=400, B=1 << 14, seed=2)
    first, last = np.mean(h[:3]), np.mean(h[-10:])
    print(f"sphere: mean percentage error {first:.3f} -> {last:.4f}")
    assert last < first / 8
