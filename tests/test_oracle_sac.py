"""Pins of the SAC oracle (oracle/sac.py) against things other than itself: scipy's normal
density plus the change of variables written out, central finite differences, an
independent float64 torch.autograd + torch.optim.Adam implementation of whole steps, the
closed-form first Adam step, and hand cases."""
import copy

import numpy as np
import torch
from scipy import stats

import workloads
from oracle import mlp, philox, sac

HP = dict(workloads.DEFAULT_HP, seed=21, target_entropy=-2.0, lr_alpha=3e-4, init_log_alpha=-0.3)


def _agent(hp=HP, O=3, A=2, hidden=(6, 5), B=7, cap=50, fill=40, data_seed=0):
    ag = sac.Agent(hp, O, A, list(hidden), B, cap)
    rng = np.random.default_rng(data_seed)
    ag.buffer.insert(rng.standard_normal((fill, O)), rng.uniform(-1, 1, (fill, A)), rng.standard_normal(fill),
                     (rng.random(fill) < 0.3).astype(np.float32), rng.standard_normal((fill, O)))
    # biases away from zero so that every path carries signal
    for net in [ag.actor] + ag.critic + ag.t_critic:
        for l, (W, b) in enumerate(net):
            b[...] = 0.1 * np.random.default_rng(100 + l).standard_normal(b.shape)
    return ag


def test_log_prob_is_the_tanh_gaussian_density():
    """log pi(a) = sum_j log N(u_j; mu_j, std_j) - sum_j log(1 - a_j^2), a = tanh(u): the normal
    density from scipy, the Jacobian of tanh written out directly."""
    rng = np.random.default_rng(1)
    B, A, O = 64, 3, 4
    net = [(np.zeros((O, 2 * A)), np.concatenate([rng.standard_normal(A), rng.uniform(-3, 1, A)]))]
    eps = rng.standard_normal((B, A))
    s = rng.standard_normal((B, O))
    a, logp, _ = sac.sample_policy(net, s, eps)
    mu, std = net[0][1][:A], np.exp(net[0][1][A:])
    u = mu + std * eps
    want = stats.norm.logpdf(u, loc=mu, scale=std).sum(axis=1) - np.log(1.0 - np.tanh(u) ** 2).sum(axis=1)
    np.testing.assert_allclose(a, np.tanh(u), rtol=1e-14)
    np.testing.assert_allclose(logp, want, rtol=1e-10, atol=1e-10)
    # far in the tails the direct Jacobian underflows; the stable form must agree with the asymptote
    # log(1 - tanh(u)^2) -> log 4 - 2|u|
    big = np.array([[30.0, -40.0, 25.0]])
    net2 = [(np.zeros((O, 2 * A)), np.concatenate([big[0], np.full(A, -20.0)]))]
    _, lp, _ = sac.sample_policy(net2, s[:1], np.zeros((1, A)))
    gauss = -(-20.0) * A - 0.5 * A * np.log(2 * np.pi)
    np.testing.assert_allclose(lp[0], gauss - np.sum(np.log(4.0) - 2 * np.abs(big)), rtol=1e-12)


def test_density_integrates_to_one_in_one_dimension():
    """Numerical integral over a in (-1, 1) of exp(log pi(a)) for A = 1, with log pi evaluated by the
    oracle at the u that produces a."""
    mu, ls = 0.3, -0.4
    net = [(np.zeros((1, 2)), np.array([mu, ls]))]
    u = np.linspace(-12, 12, 200001)
    eps = ((u - mu) / np.exp(ls))[:, None]
    a, logp, _ = sac.sample_policy(net, np.zeros((u.size, 1)), eps)
    integral = np.trapezoid(np.exp(logp), a[:, 0])
    assert abs(integral - 1.0) < 1e-6


def test_log_std_clamp_bounds_the_std_and_passes_no_gradient():
    ag = _agent()
    ag.actor[-1][1][ag.A:] = np.array([5.0, -30.0])        # both outside [-20, 2]
    s = np.random.default_rng(2).standard_normal((ag.B, ag.O)) * 1e-3
    eps = np.random.default_rng(3).standard_normal((ag.B, ag.A))
    a, logp, pc = sac.sample_policy(ag.actor, s, eps)
    np.testing.assert_allclose(pc[2], np.exp([2.0, -20.0]) * np.ones((ag.B, 1)), rtol=1e-12)
    _, g, _ = ag.actor_loss_and_grads(s, eps, 0.2)
    assert np.all(g[-1][1][ag.A:] == 0.0) and np.all(g[-1][0][:, ag.A:] == 0.0)   # log_std head gets nothing
    assert np.any(g[-1][1][:ag.A] != 0.0)


def _fd(params, loss_fn, grads, tol=2e-6, h=1e-6):
    worst = 0.0
    for (W, b), (gW, gb) in zip(params, grads):
        for arr, g in ((W, gW), (b, gb)):
            flat, gflat = arr.reshape(-1), g.reshape(-1)
            for i in range(0, flat.size, max(1, flat.size // 7)):
                old = flat[i]
                flat[i] = old + h; up = loss_fn()
                flat[i] = old - h; dn = loss_fn()
                flat[i] = old
                fd = (up - dn) / (2 * h)
                worst = max(worst, abs(fd - gflat[i]) / max(1.0, abs(fd)))
    assert worst < tol, worst


def test_actor_and_critic_gradients_match_finite_differences():
    ag = _agent()
    rng = np.random.default_rng(5)
    s = rng.standard_normal((ag.B, ag.O)); a = rng.uniform(-1, 1, (ag.B, ag.A)); y = rng.standard_normal(ag.B)
    eps = rng.standard_normal((ag.B, ag.A))
    loss, grads = ag.critic_loss_and_grads(s, a, y)
    for k in range(2):
        _fd(ag.critic[k], lambda: ag.critic_loss_and_grads(s, a, y)[0], grads[k])
    loss, g, logp = ag.actor_loss_and_grads(s, eps, 0.37)
    _fd(ag.actor, lambda: ag.actor_loss_and_grads(s, eps, 0.37)[0], g)
    # the loss itself, from its definition
    a_pi, lp, _ = sac.sample_policy(ag.actor, s, eps)
    x = np.concatenate([s, a_pi], axis=1)
    q = np.minimum(mlp.forward(ag.critic[0], x, 'linear')[0][:, 0], mlp.forward(ag.critic[1], x, 'linear')[0][:, 0])
    np.testing.assert_allclose(loss, np.mean(0.37 * lp - q), rtol=1e-13)


def test_target_hand_cases():
    ag = _agent()
    rng = np.random.default_rng(7)
    B = ag.B
    s2 = rng.standard_normal((B, ag.O)); eps2 = rng.standard_normal((B, ag.A)); r = rng.standard_normal(B)
    assert np.array_equal(ag.bellman_target(r, np.ones(B), s2, eps2, 0.5), r)                  # terminal: reward only
    a2, logp2, _ = sac.sample_policy(ag.actor, s2, eps2)
    x = np.concatenate([s2, a2], axis=1)
    q1 = mlp.forward(ag.t_critic[0], x, 'linear')[0][:, 0]; q2 = mlp.forward(ag.t_critic[1], x, 'linear')[0][:, 0]
    y0 = ag.bellman_target(r, np.zeros(B), s2, eps2, 0.0)                                      # no entropy bonus
    np.testing.assert_allclose(y0, r + ag.hp["gamma"] * np.minimum(q1, q2), rtol=1e-13)
    y = ag.bellman_target(r, np.zeros(B), s2, eps2, 0.5)
    np.testing.assert_allclose(y - y0, -ag.hp["gamma"] * 0.5 * logp2, rtol=1e-10, atol=1e-12)  # soft value: - alpha log pi
    assert (q1 < q2).any() and (q2 < q1).any()
    ag.t_critic[0] = mlp.copy_net(ag.critic[1])            # the target nets are what is used, not the online ones
    assert not np.allclose(ag.bellman_target(r, np.zeros(B), s2, eps2, 0.5), y)


def _tnet(net):
    return [(torch.tensor(W, dtype=torch.float64, requires_grad=True), torch.tensor(b, dtype=torch.float64, requires_grad=True))
            for W, b in net]


def _tf(net, x):
    h = x
    for l, (W, b) in enumerate(net):
        h = h @ W + b
        if l < len(net) - 1:
            h = torch.relu(h)
    return h


def _t_policy(actor, s, eps, A):
    out = _tf(actor, s)
    mu, ls = out[:, :A], torch.clamp(out[:, A:], -20.0, 2.0)
    dist = torch.distributions.Normal(mu, torch.exp(ls))
    u = mu + torch.exp(ls) * eps
    a = torch.tanh(u)
    logp = dist.log_prob(u).sum(dim=1) - torch.log1p(-a * a).sum(dim=1)
    return a, logp


def test_four_steps_match_torch_autograd_and_adam_on_real_shapes():
    """The whole step re-implemented with torch autograd (float64), torch.distributions for the
    density and torch.optim.Adam for every optimiser, fed with the oracle's indices and noise."""
    hp = dict(HP, lr_actor=1e-3, lr_critic=7e-4, lr_alpha=2e-3, target_entropy=-6.0, init_log_alpha=0.2)
    O, A, B = 17, 6, 64
    ag = sac.Agent(hp, O, A, [256, 256], B, 300)
    tr = workloads.transitions(0, 0, 300)
    ag.buffer.insert(**tr)
    actor, critics, targets = _tnet(ag.actor), [_tnet(c) for c in ag.critic], [_tnet(c) for c in ag.t_critic]
    log_alpha = torch.tensor([ag.log_alpha[0]], dtype=torch.float64, requires_grad=True)
    flat = lambda net: [p for Wb in net for p in Wb]
    kw = dict(betas=(ag.hp["adam_b1"], ag.hp["adam_b2"]), eps=ag.hp["adam_eps"])
    opt_a = torch.optim.Adam(flat(actor), lr=ag.hp["lr_actor"], **kw)
    opt_c = [torch.optim.Adam(flat(c), lr=ag.hp["lr_critic"], **kw) for c in critics]
    opt_al = torch.optim.Adam([log_alpha], lr=ag.hp["lr_alpha"], **kw)
    for step in range(4):
        ag.step()
        L = ag.last
        rows = ag.buffer.gather(L["idx"])
        s, a, r, d, s2 = (torch.tensor(np.asarray(x, dtype=np.float64)) for x in rows)
        e1, e2 = torch.tensor(L["eps1"]), torch.tensor(L["eps2"])
        alpha = float(torch.exp(log_alpha.detach())[0])
        with torch.no_grad():
            a2, lp2 = _t_policy(actor, s2, e2, A)
            x2 = torch.cat([s2, a2], dim=1)
            y = r + ag.hp["gamma"] * (1 - d) * (torch.minimum(_tf(targets[0], x2)[:, 0], _tf(targets[1], x2)[:, 0]) - alpha * lp2)
        x = torch.cat([s, a], dim=1)
        for k in range(2):
            opt_c[k].zero_grad()
            (((_tf(critics[k], x)[:, 0] - y) ** 2).mean()).backward()
            opt_c[k].step()
        opt_a.zero_grad()
        for c in critics:
            for p in flat(c):
                p.grad = None
        a_pi, lp = _t_policy(actor, s, e1, A)
        xa = torch.cat([s, a_pi], dim=1)
        qmin = torch.minimum(_tf(critics[0], xa)[:, 0], _tf(critics[1], xa)[:, 0])
        (alpha * lp - qmin).mean().backward()
        opt_a.step()
        opt_al.zero_grad()
        (-(torch.exp(log_alpha) * (lp.detach() + ag.hp["target_entropy"])).mean()).backward()
        opt_al.step()
        with torch.no_grad():
            for k in range(2):
                for (Wt, bt), (W, b) in zip(targets[k], critics[k]):
                    Wt.mul_(1 - ag.hp["tau"]).add_(ag.hp["tau"] * W)
                    bt.mul_(1 - ag.hp["tau"]).add_(ag.hp["tau"] * b)
        tflat = lambda net: np.concatenate([np.concatenate([W.detach().numpy().reshape(-1), b.detach().numpy().reshape(-1)]) for W, b in net])
        for name, mine, theirs in (("actor", ag.actor, actor), ("critic1", ag.critic[0], critics[0]), ("critic2", ag.critic[1], critics[1]),
                                   ("t_critic1", ag.t_critic[0], targets[0]), ("t_critic2", ag.t_critic[1], targets[1])):
            err = np.linalg.norm(mlp.flatten(mine) - tflat(theirs)) / np.linalg.norm(tflat(theirs))
            assert err < 1e-9, (step, name, err)
        assert abs(ag.log_alpha[0] - float(log_alpha.detach()[0])) < 1e-12, step


def test_temperature_moves_the_right_way_and_first_step_is_closed_form():
    ag = _agent()
    la0 = ag.log_alpha[0]
    ag.step()
    g = ag.last["alpha_grad"]
    assert np.isclose(g, -np.exp(la0) * np.mean(ag.last["logp"] + ag.hp["target_entropy"]), rtol=1e-13)
    # first Adam step from zero moments: -lr * g / (|g| + eps)
    np.testing.assert_allclose(ag.log_alpha[0] - la0, -ag.hp["lr_alpha"] * g / (abs(g) + ag.hp["adam_eps"]), rtol=1e-9)
    # entropy below its target (log pi + target > 0 on average) must raise the temperature
    lo = _agent(hp=dict(HP, target_entropy=50.0)); lo.step()
    hi = _agent(hp=dict(HP, target_entropy=-50.0)); hi.step()
    assert lo.log_alpha[0] > la0 > hi.log_alpha[0]


def test_step_order_actor_sees_updated_critics_and_targets_move_every_step():
    ag = _agent()
    before = copy.deepcopy(ag)
    ag.step()
    L = ag.last
    s = before.buffer.gather(L["idx"])[0].astype(np.float64)
    # gradient recomputed with the critics AFTER their update reproduces the step's actor gradient ...
    probe = copy.deepcopy(before); probe.critic = copy.deepcopy(ag.critic)
    _, g_after, _ = probe.actor_loss_and_grads(s, L["eps1"], L["alpha"])
    assert np.array_equal(mlp.flatten(g_after), mlp.flatten(L["actor_grads"]))
    # ... and with the critics before it does not
    _, g_before, _ = before.actor_loss_and_grads(s, L["eps1"], L["alpha"])
    assert not np.array_equal(mlp.flatten(g_before), mlp.flatten(L["actor_grads"]))
    tau = ag.hp["tau"]
    for k in range(2):                                   # Polyak towards the critics after the update, every step
        np.testing.assert_allclose(mlp.flatten(ag.t_critic[k]),
                                   (1 - tau) * mlp.flatten(before.t_critic[k]) + tau * mlp.flatten(ag.critic[k]), rtol=1e-14, atol=1e-16)
    old_t = mlp.flatten(ag.t_critic[0]).copy()
    ag.step()
    assert not np.array_equal(mlp.flatten(ag.t_critic[0]), old_t)
    assert L["alpha"] == np.exp(before.log_alpha[0])     # the temperature in force is the one from before the step


def test_noise_streams_are_distinct_and_keyed_by_step():
    ag = _agent(); ag.step(); L0 = dict(ag.last); ag.step(); L1 = ag.last
    assert not np.array_equal(L0["eps1"], L0["eps2"]) and not np.array_equal(L0["eps1"], L1["eps1"])
    assert np.array_equal(L0["eps1"], philox.normals(ag.seed, ag.B * ag.A, 0, philox.STREAM_SAC_S).reshape(ag.B, ag.A))
    assert np.array_equal(L1["eps2"], philox.normals(ag.seed, ag.B * ag.A, 1, philox.STREAM_SAC_S2).reshape(ag.B, ag.A))


def test_agent_in_population_equals_agent_alone_bit_for_bit():
    hps = [dict(h, target_entropy=-2.0) for h in workloads.hparams(2, P=3)]
    def build(hp_list, agents):
        pop = sac.Population(hp_list, 3, 2, [8, 8], 16, 64)
        for j, i in enumerate(agents):
            pop.insert(j, **workloads.transitions(2, i, 50, obs_dim=3, act_dim=2))
        pop.update(3)
        return pop
    full = build(hps, range(3))
    for i in (0, 2):
        alone = build([hps[i]], [i])
        for which in sac.WHICH[:14]:
            assert np.array_equal(full.get_params(i, which), alone.get_params(0, which)), (i, which)
