"""Adam and Polyak averaging for the oracle (test infrastructure only).

The paper's update is "a variant of stochastic gradient descent" (Sec. 1) with
the standard hyperparametrization of the cited TD3/SAC implementations
(Sec. 4.1); both use Adam (Kingma & Ba 2015) and soft target updates.

Pins: tests/test_oracle_optim.py (closed-form first step from zero moments,
torch.optim.Adam in float64 over several steps, Polyak identities).
"""
import numpy as np


class AdamState:
    """First and second moment for one network (same list-of-pairs shape)."""

    def __init__(self, net):
        self.m = [(np.zeros_like(W), np.zeros_like(b)) for W, b in net]
        self.v = [(np.zeros_like(W), np.zeros_like(b)) for W, b in net]


def adam_step(net, grads, state, lr, t, b1, b2, eps):
    """One Adam step in place; t is the 1-based count of steps including this
    one.  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
    theta <- theta - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)."""
    c1 = 1.0 - float(b1) ** t
    c2 = 1.0 - float(b2) ** t
    for l in range(len(net)):
        for j in range(2):
            g = grads[l][j]
            m = state.m[l][j]
            v = state.v[l][j]
            m *= b1
            m += (1.0 - b1) * g
            v *= b2
            v += (1.0 - b2) * (g * g)
            net[l][j][...] = net[l][j] - lr * (m / c1) / (np.sqrt(v / c2) + eps)


def polyak(target, online, tau):
    """theta' <- (1 - tau) theta' + tau theta, in place on target."""
    for (Wt, bt), (W, b) in zip(target, online):
        Wt[...] = (1.0 - tau) * Wt + tau * W
        bt[...] = (1.0 - tau) * bt + tau * b
