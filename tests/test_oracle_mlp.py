"""Pins for oracle/mlp.py: finite differences, torch.autograd (float64),
torch.bmm for the population layer of App. C, and init statistics."""
import numpy as np
import torch

from oracle import mlp


def _rand_net(rng, sizes):
    return [(rng.standard_normal((i, o)) * 0.7, rng.standard_normal(o) * 0.3)
            for i, o in zip(sizes[:-1], sizes[1:])]


def _to_torch(net):
    return [(torch.tensor(W, requires_grad=True), torch.tensor(b, requires_grad=True)) for W, b in net]


def _torch_forward(tnet, x, head):
    h = x
    for l, (W, b) in enumerate(tnet):
        h = h @ W + b
        if l < len(tnet) - 1:
            h = torch.relu(h)
        elif head == 'tanh':
            h = torch.tanh(h)
    return h


def test_layer_is_batched_matmul_plus_bias():
    # App. C: x[P,B,in].matmul(W[P,in,out]) + b[P,1,out]
    rng = np.random.default_rng(0)
    P, B, I, O = 3, 5, 7, 4
    W = rng.standard_normal((P, I, O)); b = rng.standard_normal((P, 1, O)); x = rng.standard_normal((P, B, I))
    ref = (torch.bmm(torch.tensor(x), torch.tensor(W)) + torch.tensor(b)).numpy()
    for p in range(P):
        y, _ = mlp.forward([(W[p], b[p, 0])], x[p], 'linear')
        np.testing.assert_allclose(y, ref[p], rtol=1e-13, atol=1e-13)


def test_forward_and_backward_match_torch_autograd_on_real_shapes():
    rng = np.random.default_rng(1)
    for sizes, head in (([17, 256, 256, 6], 'tanh'), ([23, 256, 256, 1], 'linear')):
        net = _rand_net(rng, sizes)
        for W, _ in net:
            W *= 0.1
        x = rng.standard_normal((256, sizes[0]))
        dy = rng.standard_normal((256, sizes[-1]))
        y, cache = mlp.forward(net, x, head)
        grads, dx = mlp.backward(net, cache, dy, need_dx=True)
        tnet = _to_torch(net)
        tx = torch.tensor(x, requires_grad=True)
        ty = _torch_forward(tnet, tx, head)
        np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-12, atol=1e-12)
        (ty * torch.tensor(dy)).sum().backward()
        for (gW, gb), (tW, tb) in zip(grads, tnet):
            np.testing.assert_allclose(gW, tW.grad.numpy(), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(gb, tb.grad.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_backward_matches_central_finite_differences_on_tiny_nets():
    rng = np.random.default_rng(2)
    for sizes, head in (([3, 4, 4, 2], 'tanh'), ([5, 4, 4, 1], 'linear'), ([3, 2], 'tanh')):
        net = _rand_net(rng, sizes)
        x = rng.standard_normal((5, sizes[0]))
        c = rng.standard_normal((5, sizes[-1]))           # L = sum(c * y)
        y, cache = mlp.forward(net, x, head)
        grads, dx = mlp.backward(net, cache, c, need_dx=True)
        h = 1e-6

        def L():
            return float(np.sum(c * mlp.forward(net, x, head)[0]))
        for l, (W, b) in enumerate(net):
            for arr, g in ((W, grads[l][0]), (b, grads[l][1])):
                it = np.nditer(arr, flags=['multi_index'])
                for _ in it:
                    i = it.multi_index
                    old = arr[i]
                    arr[i] = old + h; lp = L()
                    arr[i] = old - h; lm = L()
                    arr[i] = old
                    fd = (lp - lm) / (2 * h)
                    assert abs(fd - g[i]) <= 1e-6 * max(1.0, abs(fd)), (sizes, l, i, fd, g[i])
        for i in np.ndindex(x.shape):
            old = x[i]
            x[i] = old + h; lp = L()
            x[i] = old - h; lm = L()
            x[i] = old
            assert abs((lp - lm) / (2 * h) - dx[i]) <= 1e-6 * max(1.0, abs(dx[i]))


def test_relu_gradient_is_zero_at_and_below_zero():
    net = [(np.array([[1.0, -1.0, 0.0]]), np.zeros(3)), (np.ones((3, 1)), np.zeros(1))]
    x = np.array([[2.0]])                                  # pre-activations 2, -2, 0
    y, cache = mlp.forward(net, x, 'linear')
    grads, _ = mlp.backward(net, cache, np.ones((1, 1)))
    assert grads[0][1].tolist() == [1.0, 0.0, 0.0]


def test_glorot_init_statistics_and_fp32_exactness():
    net = mlp.init_mlp(42, mlp.NET_ACTOR, [17, 256, 256, 6])
    for (W, b), (fi, fo) in zip(net, ((17, 256), (256, 256), (256, 6))):
        lim = np.sqrt(6.0 / (fi + fo))
        assert np.all(b == 0)
        assert np.abs(W).max() <= lim * (1 + 1e-6)
        assert np.array_equal(W, W.astype(np.float32).astype(np.float64))   # fp32 values
        if W.size > 4000:
            assert abs(W.mean()) < 4 * lim / np.sqrt(3 * W.size)
            assert abs(W.var() - lim ** 2 / 3) < 0.05 * lim ** 2 / 3
    other = mlp.init_mlp(43, mlp.NET_ACTOR, [17, 256, 256, 6])
    c1 = mlp.init_mlp(42, mlp.NET_CRITIC1, [23, 256, 256, 1])
    c2 = mlp.init_mlp(42, mlp.NET_CRITIC2, [23, 256, 256, 1])
    assert np.mean(net[1][0] == other[1][0]) < 0.01
    assert np.mean(c1[1][0] == c2[1][0]) < 0.01
    assert np.mean(net[1][0] == c1[1][0]) < 0.01
    # layers of one net use different sub-streams
    assert np.mean(net[1][0][:17] == net[0][0]) < 0.01


def test_flatten_order_is_layerwise_weights_then_bias():
    net = [(np.arange(6.0).reshape(2, 3), np.array([10., 11., 12.])), (np.array([[20.], [21.], [22.]]), np.array([30.]))]
    assert mlp.flatten(net).tolist() == [0, 1, 2, 3, 4, 5, 10, 11, 12, 20, 21, 22, 30]
