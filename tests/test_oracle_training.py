"""Pins for the oracle's training-loop pieces: training mask on the loss and Adam (Section 4)."""
import numpy as np

from oracle import bns_oracle as orc


def test_masked_loss_equals_loss_on_the_training_subset():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((50, 7))
    y = rng.integers(0, 7, size=50)
    mask = rng.random(50) < 0.4
    ym = np.where(mask, y, -1)
    loss, g = orc.loss_and_grad(z, ym, 0)
    loss_sub, g_sub = orc.loss_and_grad(z[mask], y[mask], 0)
    np.testing.assert_allclose(loss, loss_sub, rtol=1e-14)
    np.testing.assert_allclose(g[mask], g_sub, rtol=1e-14)
    assert np.all(g[~mask] == 0)
    # multi-label: masked entries
    yb = (rng.random((50, 7)) < 0.3).astype(np.uint8)
    mb = rng.random((50, 7)) < 0.5
    lossb, gb = orc.loss_and_grad(z, np.where(mb, yb, 255).astype(np.uint8), 1)
    full_l, full_g = orc.loss_and_grad(z, yb, 1)
    sig = 1 / (1 + np.exp(-z))
    terms = -(yb * np.log(sig) + (1 - yb) * np.log(1 - sig))
    np.testing.assert_allclose(lossb, terms[mb].sum(), rtol=1e-12)
    np.testing.assert_allclose(gb[mb], full_g[mb], rtol=1e-14)
    assert np.all(gb[~mb] == 0)


def test_adam_constant_gradient_closed_form():
    """With a constant gradient the bias-corrected moments equal g and g^2 at every step, so each
    step moves every weight by lr * g / (|g| + eps)."""
    g = np.array([0.5, -2.0, 1e-3])
    W, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    lr, eps = 0.01, 1e-8
    for t in range(1, 6):
        W, m, v = orc.adam_step(W, g, m, v, lr, 0.9, 0.999, eps, t)
        np.testing.assert_allclose(W, -t * lr * g / (np.abs(g) + eps), rtol=1e-12)


def test_adam_matches_the_library_optimiser():
    import torch
    rng = np.random.default_rng(1)
    W0 = rng.standard_normal((6, 5))
    grads = [rng.standard_normal((6, 5)) for _ in range(7)]
    wt = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([wt], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    W, m, v = W0.copy(), np.zeros_like(W0), np.zeros_like(W0)
    for t, g in enumerate(grads, start=1):
        wt.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        W, m, v = orc.adam_step(W, g, m, v, 0.01, 0.9, 0.999, 1e-8, t)
        np.testing.assert_allclose(W, wt.detach().numpy(), rtol=1e-12, atol=1e-14)
