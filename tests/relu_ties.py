"""ReLU ties: showing that a gradient difference between the fp32 device path and the fp64 oracle is one hidden
unit resolved the other way, not an error.

A hidden pre-activation z = h W + b that lies within the fp32 rounding error of its own sum is positive on one
side and non-positive on the other.  The forward value changes by |z| (nothing), but the unit's ReLU mask enters
or leaves the backward pass, which changes the gradient by that sample's share of the unit (about 1e-3 of the
gradient's norm at a batch of 256).  Both results are correct TD3 steps.  The functions here recompute the
oracle's gradient of one network with chosen masks flipped (by negating the stored pre-activation before calling
the oracle's own backward) and search the near-tie units for the set of flips that reproduces the device's gradient.

The size of "near": the rounding error of an fp32 dot product is bounded by its length times 2^-24 times the sum
of the absolute values of its terms, so a unit's margin is measured as rho = |z| / (|h| |W| + |b|).
"""
import numpy as np

from oracle import mlp


def relative_margins(net, cache):
    """Per hidden layer l: rho[l][b, j] = |z| / (|h_in| |W| + |b|) for the hidden pre-activations of a forward pass."""
    inputs, pre = cache[0], cache[1]
    out = []
    for l in range(len(net) - 1):
        W, b = net[l]
        scale = np.abs(inputs[l]) @ np.abs(W) + np.abs(b)
        out.append(np.abs(pre[l]) / np.maximum(scale, 1e-300))
    return out


def smallest_margin(net, cache):
    return min(float(r.min()) for r in relative_margins(net, cache))


def candidates(nets_and_caches, rho_max, limit):
    """[(rho, which pass, layer, row, unit)] of the hidden units closest to their kink, ascending, at most `limit`."""
    found = []
    for p, (net, cache) in enumerate(nets_and_caches):
        for l, rho in enumerate(relative_margins(net, cache)):
            rows, units = np.nonzero(rho < rho_max)
            found += [(float(rho[r, u]), p, l, int(r), int(u)) for r, u in zip(rows, units)]
    found.sort()
    return found[:limit]


def flip(cache, layer, row, unit):
    """Resolve one hidden unit the other way (in place): the sign of its stored pre-activation decides the mask in
    mlp.backward; its magnitude is below anything the gradient can see."""
    z = cache[1][layer][row, unit]
    cache[1][layer][row, unit] = -z if z != 0.0 else 1e-300


def unflatten(flat, fan_in, fan_out, hidden=(256, 256)):
    """Inverse of mlp.flatten: canonical flat vector -> [(W, b)] (fp64 copies)."""
    sizes = [fan_in] + list(hidden) + [fan_out]
    net, o = [], 0
    flat = np.asarray(flat, dtype=np.float64)
    for fi, fo in zip(sizes[:-1], sizes[1:]):
        W = flat[o:o + fi * fo].reshape(fi, fo).copy(); o += fi * fo
        b = flat[o:o + fo].copy(); o += fo
        net.append((W, b))
    assert o == flat.size
    return net


KAPPA = 0.01      # an activation carries the rounding error of its own dot product; measured in units of the gradient's
                  # error bound (parity_checks.ETA times the sum of absolute terms) that is KAPPA times the activation's
                  # own sum of absolute terms: 4e-8 of it, where an fp32 dot product of n terms errs by about
                  # 2^-24 sqrt(n) times its rms term.  Matters at first-layer fan-ins of several hundred.


def abs_sums(net, cache, dy, need_dx=False):
    """Running error scale of a backward pass: the oracle's backward with every product taken on absolute values.
    For every gradient entry (canonical flat order) this is the sum of the absolute values of all the terms that
    enter it, including those of the backward products upstream of it (D_l = D_{l+1} |W_{l+1}|^T under the ReLU
    mask, dW_l -> (|in_l| + KAPPA A_l)^T D_l with A_l the same kind of sum for the forward pass that produced in_l,
    db_l -> column sums of D_l): the scale of the rounding error of an fp32 evaluation of that entry, cancellation in
    the back-propagated signal included.  Used for tolerances only; reference values always come from the oracle's
    own backward.  Returns (flat scale, D at the input or None)."""
    inputs, pre, y, head = cache
    last = len(net) - 1
    A = [np.zeros_like(inputs[0])]                      # the network's input is exact
    for l in range(last):
        a = (np.abs(inputs[l]) + A[l]) @ np.abs(net[l][0]) + np.abs(net[l][1])
        A.append(a * (pre[l] > 0.0))
    out = [None] * len(net)
    d = np.abs(dy)
    for l in range(last, -1, -1):
        if l == last:
            dz = d * (1.0 - y * y) if head == 'tanh' else d
        else:
            dz = d * (pre[l] > 0.0)
        out[l] = ((np.abs(inputs[l]) + KAPPA * A[l]).T @ dz, dz.sum(axis=0))
        if l > 0 or need_dx:
            d = dz @ np.abs(net[l][0]).T
    return mlp.flatten(out), (d if need_dx else None)


class _Pass:
    """One gradient of one network as the oracle computes it, with the forward caches open to flips.
    passes: [(net, cache)] whose hidden units are candidates; gradient(): flat gradient under the current masks;
    noise_scale(): abs_sums of the same gradient."""

    def flip(self, p, layer, row, unit):
        flip(self.passes[p][1], layer, row, unit)


class CriticPass(_Pass):
    """Critic k of a TD3 or SAC agent on the batch of the step just taken (ag.last holds its indices and Bellman
    targets), from the critic as it was before the step.  scale: factor on the loss (1/P with shared critics)."""

    def __init__(self, ag, critic_before, scale=1.0):
        s, a = (x.astype(np.float64) for x in ag.buffer.gather(ag.last["idx"])[:2])
        self.net = critic_before
        x = np.concatenate([s, a], axis=1)
        q, self.cache = mlp.forward(self.net, x, 'linear')
        self.dy = (scale * 2.0 * (q[:, 0] - ag.last["y"]) / x.shape[0])[:, None]
        self.passes = [(self.net, self.cache)]

    def gradient(self):
        g, _ = mlp.backward(self.net, self.cache, self.dy)
        return mlp.flatten(g)

    def noise_scale(self):
        return abs_sums(self.net, self.cache, self.dy)[0]


class SharedCriticPass(_Pass):
    """Shared critic k: the mean over the population of the agents' critic gradients.  A flip touches one agent's
    pass only, so the per-agent gradients are kept and only that one is recomputed."""

    def __init__(self, agents, critic_before):
        P = len(agents)
        self.parts = [CriticPass(ag, critic_before, scale=1.0 / P) for ag in agents]
        self.passes = [ps.passes[0] for ps in self.parts]
        self.grads = [None] * P

    def flip(self, p, layer, row, unit):
        flip(self.passes[p][1], layer, row, unit)
        self.grads[p] = None

    def gradient(self):
        for p, ps in enumerate(self.parts):
            if self.grads[p] is None:
                self.grads[p] = ps.gradient()
        return np.sum(self.grads, axis=0)

    def noise_scale(self):
        return np.sum([ps.noise_scale() for ps in self.parts], axis=0)


class ActorPass(_Pass):
    """Actor phase of a TD3 agent: actor as it was before the step, critic 1 as it is after its update
    (ag.critic[0] unless another one is given)."""

    def __init__(self, ag, actor_before, critic_after=None):
        s = ag.buffer.gather(ag.last["idx"])[0].astype(np.float64)
        self.O, self.actor = ag.O, actor_before
        self.critic = ag.critic[0] if critic_after is None else critic_after
        a_pi, self.a_cache = mlp.forward(self.actor, s, 'tanh')
        _, self.c_cache = mlp.forward(self.critic, np.concatenate([s, a_pi], axis=1), 'linear')
        self.B = s.shape[0]
        self.passes = [(self.actor, self.a_cache), (self.critic, self.c_cache)]

    def gradient(self):
        _, dx = mlp.backward(self.critic, self.c_cache, np.full((self.B, 1), -1.0 / self.B), need_dx=True)
        g, _ = mlp.backward(self.actor, self.a_cache, dx[:, self.O:])
        return mlp.flatten(g)

    def noise_scale(self):
        _, dx = abs_sums(self.critic, self.c_cache, np.full((self.B, 1), 1.0 / self.B), need_dx=True)
        return abs_sums(self.actor, self.a_cache, dx[:, self.O:])[0]


class SacActorPass(_Pass):
    """Actor phase of a SAC agent: (1/B) sum [alpha log pi(a|s) - min_k Q_k(s, a)] through both critics as they are
    after their update (or the ones given), actor as before the step, noise and alpha of the step from ag.last."""

    def __init__(self, ag, actor_before, critics_after=None):
        from oracle import sac
        self.sac = sac
        s = ag.buffer.gather(ag.last["idx"])[0].astype(np.float64)
        self.O, self.B, self.actor = ag.O, s.shape[0], actor_before
        self.critics = list(ag.critic) if critics_after is None else critics_after
        self.alpha = ag.last["alpha"]
        a, _, self.pcache = sac.sample_policy(self.actor, s, ag.last["eps1"])
        x = np.concatenate([s, a], axis=1)
        self.q, self.c_caches = [], []
        for k in range(2):
            qk, ck = mlp.forward(self.critics[k], x, 'linear')
            self.q.append(qk[:, 0]); self.c_caches.append(ck)
        self.passes = [(self.actor, self.pcache[0]), (self.critics[0], self.c_caches[0]), (self.critics[1], self.c_caches[1])]

    def _d_a(self):
        first = self.q[0] <= self.q[1]
        d_a = 0.0
        for k, sel in ((0, first), (1, ~first)):
            _, dx = mlp.backward(self.critics[k], self.c_caches[k], (-1.0 / self.B * sel)[:, None], need_dx=True)
            d_a = d_a + dx[:, self.O:]
        return d_a

    def gradient(self):
        return mlp.flatten(self.sac.policy_backward(self.actor, self.pcache, self._d_a(), np.full(self.B, self.alpha / self.B)))

    def noise_scale(self):
        # the seed of the actor's backward pass, as policy_backward forms it: (d_mu, d_log_std)
        cache, a, std, eps, inside = self.pcache
        d_logp = np.full(self.B, self.alpha / self.B)
        first = self.q[0] <= self.q[1]
        d_a = 0.0
        for k, sel in ((0, first), (1, ~first)):
            d_a = d_a + abs_sums(self.critics[k], self.c_caches[k], (1.0 / self.B * sel)[:, None], need_dx=True)[1][:, self.O:]
        d_u = d_a * (1.0 - a * a) + np.abs(d_logp[:, None] * 2.0 * a)
        d_ls = (d_u * np.abs(std * eps) + np.abs(d_logp[:, None])) * inside
        return abs_sums(self.actor, cache, np.concatenate([d_u, d_ls], axis=1))[0]


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


RHO_TIE = 1e-6     # a unit counts as "on its kink" below this relative margin (fp32 dot products of <= 448 terms:
                   # the rounding bound is n * 2^-24 = 2.7e-5 of the sum of absolute terms, the observed error ~1e-7)


def explain(pass_, g_device, rho_max=RHO_TIE, limit=32, goal=1e-5):
    """Greedy search over the units nearest their kink: keep a flip if it brings the oracle's gradient closer to the
    device's; passes over the candidates are repeated while one of them still helps.  Returns (error before, error after, [(rho, pass, layer, row, unit)] kept, smallest rho seen)."""
    base = rel_l2(g_device, pass_.gradient())
    cands = candidates(pass_.passes, rho_max, limit)
    kept, err = [], base
    progress = True
    while progress and err > goal:                        # again over those left: a small flip shows once a large one is out of the way
        progress = False
        for c in cands:
            if err <= goal:
                break
            if c in kept:
                continue
            _, p, l, r, u = c
            pass_.flip(p, l, r, u)
            e = rel_l2(g_device, pass_.gradient())
            if e < 0.7 * err:
                kept.append(c); err = e
                progress = True
            else:
                pass_.flip(p, l, r, u)
    return base, err, kept, (cands[0][0] if cands else float("inf"))


def redo_adam(before, g_flat, shape, lr, b1, b2, eps, count, tau=None):
    """The oracle's own Adam (and Polyak) applied to the state `before` (dict of flat 'theta', 'm', 'v', 'target')
    with the gradient g_flat: what the oracle's step gives when its masks are the ones behind g_flat."""
    from oracle import optim
    net = unflatten(before["theta"], *shape)
    st = optim.AdamState(net)
    st.m, st.v = unflatten(before["m"], *shape), unflatten(before["v"], *shape)
    optim.adam_step(net, unflatten(g_flat, *shape), st, lr, count, b1, b2, eps)
    out = {"theta": mlp.flatten(net), "m": mlp.flatten(st.m), "v": mlp.flatten(st.v), "g": np.asarray(g_flat, dtype=np.float64)}
    if tau is not None:
        tgt = unflatten(before["target"], *shape)
        optim.polyak(tgt, net, tau)
        out["target"] = mlp.flatten(tgt)
    return out


def tie_envelope(pass_, skip=(), rho_max=RHO_TIE, limit=32):
    """Per gradient entry, how far the hidden units still on their kink (relative margin < rho_max, those in `skip`
    excepted) can move it: the sum over those units of |gradient with the unit flipped - gradient|.  A flip too
    small to show in the gradient's norm (one sample's share of one first-layer unit, say) cannot be told from
    rounding, so the element-wise comparison allows for it.  Returns (flat array, number of units)."""
    g0 = pass_.gradient()
    env = np.zeros_like(g0)
    cands = [c for c in candidates(pass_.passes, rho_max, limit) if c not in skip]
    for _, p, l, r, u in cands:
        pass_.flip(p, l, r, u)
        env += np.abs(pass_.gradient() - g0)
        pass_.flip(p, l, r, u)
    return env, len(cands)
