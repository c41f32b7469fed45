"""MLP forward and hand-derived backward for the oracle (test infrastructure).

Sec. 4.1 of the paper: actors and critics are fully connected networks; App. C
fixes the layer as y = x W + b with W stored [in, out].  Hidden activations are
ReLU; the actor head is tanh (actions in [-1, 1]) and the critic head is
linear.  The appendix listing puts a ReLU after the last layer too; that is
read as a simplification of the example and not followed.

A network is a list of (W, b) pairs, W of shape [in, out], b of shape [out].
Everything here is fp64 unless the caller passes another dtype.

Pins: tests/test_oracle_mlp.py (central finite differences on tiny nets,
torch.autograd in float64 on the real shapes, torch.bmm for the layer).
"""
import numpy as np

from . import philox

NET_ACTOR = 0
NET_CRITIC1 = 1
NET_CRITIC2 = 2


def glorot_limit(fan_in, fan_out):
    """sqrt(6 / (fan_in + fan_out)) evaluated in fp32 (division, then square
    root, both correctly rounded), so that the initial weights can be equal bit
    for bit on any IEEE machine."""
    return np.sqrt(np.float32(6.0) / np.float32(fan_in + fan_out), dtype=np.float32)


def init_mlp(seed, net_id, sizes, dtype=np.float64):
    """Glorot-uniform weights, zero biases (reading: the benchmark configs ask
    for Glorot-uniform; the appendix listing's Kaiming init is not used).

    Weight e (row-major flat index in [in, out]) of layer l is
    (2u - 1) * limit, u = top 24 bits of word e of stream 4 with
    sub = 16*net_id + l; computed in fp32, then widened."""
    net = []
    for l, (fi, fo) in enumerate(zip(sizes[:-1], sizes[1:])):
        w = philox.words(seed, fi * fo, 0, philox.STREAM_INIT, 16 * net_id + l)
        u = ((w >> np.uint32(8)).astype(np.float32)) * np.float32(2.0 ** -24)
        centred = np.float32(2.0) * u - np.float32(1.0)          # exact in fp32
        W = (centred * glorot_limit(fi, fo)).astype(np.float32)  # one rounding
        net.append((W.reshape(fi, fo).astype(dtype), np.zeros(fo, dtype=dtype)))
    return net


def copy_net(net):
    return [(W.copy(), b.copy()) for W, b in net]


def forward(net, x, head):
    """Return (y, cache).  head is 'tanh' or 'linear'.  cache keeps each
    layer's input and the hidden pre-activations for backward()."""
    inputs, pre = [], []
    h = x
    last = len(net) - 1
    for l, (W, b) in enumerate(net):
        inputs.append(h)
        z = h @ W + b
        pre.append(z)
        if l < last:
            h = np.maximum(z, 0.0)
        elif head == 'tanh':
            h = np.tanh(z)
        elif head == 'linear':
            h = z
        else:
            raise ValueError(head)
    return h, (inputs, pre, h, head)


def backward(net, cache, dy, need_dx=False):
    """Given dL/dy, return ([(dW, db)], dL/dx or None).

    Derivation, layer by layer from the top: dz = dy * act'(z);
    dW = input^T dz; db = column sums of dz; d(input) = dz W^T.
    ReLU'(z) is 1 for z > 0 and 0 otherwise (0 at exactly 0);
    tanh'(z) = 1 - tanh(z)^2."""
    inputs, pre, y, head = cache
    grads = [None] * len(net)
    last = len(net) - 1
    d = dy
    for l in range(last, -1, -1):
        if l == last:
            dz = d * (1.0 - y * y) if head == 'tanh' else d
        else:
            dz = d * (pre[l] > 0.0)
        grads[l] = (inputs[l].T @ dz, dz.sum(axis=0))
        if l > 0 or need_dx:
            d = dz @ net[l][0].T
    return grads, (d if need_dx else None)


def flatten(net_or_grads):
    """Canonical export order: layer by layer, W row-major [in, out] then b."""
    return np.concatenate([np.concatenate([W.reshape(-1), b.reshape(-1)])
                           for W, b in net_or_grads])
