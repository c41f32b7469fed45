"""Pins for oracle/optim.py."""
import numpy as np
import torch

from oracle import optim


def _net(rng):
    return [(rng.standard_normal((4, 3)), rng.standard_normal(3)), (rng.standard_normal((3, 2)), rng.standard_normal(2))]


def test_first_adam_step_from_zero_moments_is_closed_form():
    # m_hat = g, v_hat = g^2  =>  delta = -lr * g / (|g| + eps)
    rng = np.random.default_rng(0)
    net = _net(rng)
    before = [(W.copy(), b.copy()) for W, b in net]
    grads = [(rng.standard_normal(W.shape) * 10.0 ** rng.integers(-9, 2, W.shape), rng.standard_normal(b.shape)) for W, b in net]
    grads[0][0][0, 0] = 0.0
    st = optim.AdamState(net)
    lr, eps = 3e-4, 1e-8
    optim.adam_step(net, grads, st, lr, 1, 0.9, 0.999, eps)
    for l in range(2):
        for j in range(2):
            g = grads[l][j]
            np.testing.assert_allclose(net[l][j] - before[l][j], -lr * g / (np.abs(g) + eps), rtol=1e-9, atol=1e-18)
    assert net[0][0][0, 0] == before[0][0][0, 0]           # zero gradient, zero change


def test_adam_matches_torch_optim_over_ten_steps():
    rng = np.random.default_rng(1)
    net = _net(rng)
    tparams = [torch.tensor(a.copy(), requires_grad=True) for W, b in net for a in (W, b)]
    opt = torch.optim.Adam(tparams, lr=7e-4, betas=(0.9, 0.999), eps=1e-8)
    st = optim.AdamState(net)
    for t in range(1, 11):
        grads = [(rng.standard_normal(W.shape), rng.standard_normal(b.shape)) for W, b in net]
        flat = [a for g in grads for a in g]
        for p, g in zip(tparams, flat):
            p.grad = torch.tensor(g.copy())
        opt.step()
        optim.adam_step(net, grads, st, 7e-4, t, 0.9, 0.999, 1e-8)
    flat_net = [a for W, b in net for a in (W, b)]
    for p, a in zip(tparams, flat_net):
        np.testing.assert_allclose(a, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_polyak_identities():
    rng = np.random.default_rng(2)
    online = _net(rng)
    # identical nets stay identical for any tau
    for tau in (0.0, 0.005, 0.3, 1.0):
        target = [(W.copy(), b.copy()) for W, b in online]
        optim.polyak(target, online, tau)
        for (Wt, bt), (W, b) in zip(target, online):
            np.testing.assert_allclose(Wt, W, rtol=1e-15); np.testing.assert_allclose(bt, b, rtol=1e-15)
    start = _net(rng)
    t0 = [(W.copy(), b.copy()) for W, b in start]
    optim.polyak(t0, online, 0.0)                           # tau = 0 freezes
    assert all(np.array_equal(a, b) for x, y in zip(t0, start) for a, b in zip(x, y))
    t1 = [(W.copy(), b.copy()) for W, b in start]
    optim.polyak(t1, online, 1.0)                           # tau = 1 copies
    assert all(np.array_equal(a, b) for x, y in zip(t1, online) for a, b in zip(x, y))
    # k applications with rate tau leave (1-tau)^k of the distance
    tk = [(W.copy(), b.copy()) for W, b in start]
    for _ in range(5):
        optim.polyak(tk, online, 0.25)
    for (Wt, _), (W0, _), (W, _) in zip(tk, start, online):
        np.testing.assert_allclose(Wt - W, 0.75 ** 5 * (W0 - W), rtol=1e-12, atol=1e-15)
