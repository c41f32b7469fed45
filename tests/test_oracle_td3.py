"""Pins for oracle/td3.py: the step as a whole and its pieces."""
import copy

import numpy as np
import torch

import workloads
from oracle import mlp, philox, td3

HP = dict(workloads.DEFAULT_HP, seed=11)


def _agent(hp=HP, O=3, A=2, hidden=(4, 4), B=5, cap=50, fill=40, data_seed=0):
    ag = td3.Agent(hp, O, A, list(hidden), B, cap)
    rng = np.random.default_rng(data_seed)
    ag.buffer.insert(rng.standard_normal((fill, O)), rng.uniform(-1, 1, (fill, A)), rng.standard_normal(fill),
                     (rng.random(fill) < 0.3).astype(np.float32), rng.standard_normal((fill, O)))
    return ag


def _batch(ag, t):
    idx = philox.sample_indices(ag.seed, t, ag.B, ag.buffer.count)
    return [x.astype(np.float64) for x in ag.buffer.gather(idx)]


# ---- Bellman target: hand cases ------------------------------------------------
def _const_critic(net, value):
    for W, b in net:
        W[...] = 0.0; b[...] = 0.0
    net[-1][1][...] = value


def test_target_hand_cases():
    ag = _agent()
    s, a, r, d, s2 = _batch(ag, 0)
    _const_critic(ag.t_critic[0], 1.5)
    _const_critic(ag.t_critic[1], -2.0)
    at = np.zeros((ag.B, ag.A))
    y = ag.bellman_target(r, d, s2, at)
    g = ag.hp["gamma"]
    np.testing.assert_allclose(y, r + g * (1 - d) * (-2.0), rtol=1e-14)      # min picks the smaller
    _const_critic(ag.t_critic[1], 3.0)
    np.testing.assert_allclose(ag.bellman_target(r, d, s2, at), r + g * (1 - d) * 1.5, rtol=1e-14)
    np.testing.assert_allclose(ag.bellman_target(r, np.ones_like(d), s2, at), r, rtol=0)   # done => y = r
    ag.hp["gamma"] = 0.0
    np.testing.assert_allclose(ag.bellman_target(r, d, s2, at), r, rtol=0)                 # gamma 0 => y = r


def test_target_policy_smoothing_hand_cases():
    ag = _agent()
    s2 = np.random.default_rng(3).standard_normal((5, 3))
    mu, _ = mlp.forward(ag.t_actor, s2, 'tanh')
    eps = np.random.default_rng(4).standard_normal((5, 2))
    ag.hp["policy_noise"] = 0.0
    np.testing.assert_array_equal(ag.target_action(s2, eps), mu)             # sigma 0 => mu'
    ag.hp["policy_noise"], ag.hp["noise_clip"] = 1e6, 0.125                  # noise saturates at +-c
    np.testing.assert_allclose(ag.target_action(s2, eps), np.clip(mu + 0.125 * np.sign(eps), -1, 1), rtol=1e-15)
    ag.hp["noise_clip"] = 1e6                                                # then the action at +-1
    np.testing.assert_array_equal(ag.target_action(s2, eps), np.sign(eps))
    ag.hp["policy_noise"], ag.hp["noise_clip"] = 0.2, 0.5
    out = ag.target_action(s2, eps)
    assert np.all(np.abs(out) <= 1.0) and np.all(np.abs(out - mu) <= 0.5 + 1e-15)


# ---- gradients of both losses: finite differences on a tiny agent ---------------
def _fd_check(nets_to_perturb, loss_fn, grads, tol=1e-6):
    h = 1e-6
    for net, g in zip(nets_to_perturb, grads):
        for l, (W, b) in enumerate(net):
            for arr, ga in ((W, g[l][0]), (b, g[l][1])):
                for i in np.ndindex(arr.shape):
                    old = arr[i]
                    arr[i] = old + h; lp = loss_fn()
                    arr[i] = old - h; lm = loss_fn()
                    arr[i] = old
                    fd = (lp - lm) / (2 * h)
                    assert abs(fd - ga[i]) <= tol * max(1.0, abs(fd)), (l, i, fd, ga[i])


def test_critic_and_actor_gradients_match_finite_differences():
    ag = _agent()
    for net in [ag.actor] + ag.critic:                     # make biases non-zero
        for _, b in net:
            b += 0.1
    s, a, r, d, s2 = _batch(ag, 0)
    y = np.random.default_rng(5).standard_normal(ag.B)
    _, cg = ag.critic_loss_and_grads(s, a, y)
    _fd_check(ag.critic, lambda: ag.critic_loss_and_grads(s, a, y)[0], cg)
    _, agr = ag.actor_loss_and_grads(s)
    _fd_check([ag.actor], lambda: ag.actor_loss_and_grads(s)[0], [agr])


# ---- whole step against torch autograd + torch.optim.Adam in float64 -------------
def _tnet(net):
    return [(torch.tensor(W.copy(), requires_grad=True), torch.tensor(b.copy(), requires_grad=True)) for W, b in net]


def _tf(net, x, head):
    h = x
    for l, (W, b) in enumerate(net):
        h = h @ W + b
        h = torch.relu(h) if l < len(net) - 1 else (torch.tanh(h) if head == 'tanh' else h)
    return h


def test_five_steps_match_torch_autograd_and_adam_on_real_shapes():
    hp = dict(HP, seed=5, lr_actor=1e-3, lr_critic=5e-4, tau=0.01)
    ag = _agent(hp, O=17, A=6, hidden=(256, 256), B=256, cap=3000, fill=2000)
    actor, c1, c2 = _tnet(ag.actor), _tnet(ag.critic[0]), _tnet(ag.critic[1])
    ta, tc1, tc2 = _tnet(ag.t_actor), _tnet(ag.t_critic[0]), _tnet(ag.t_critic[1])
    flat = lambda net: [p for Wb in net for p in Wb]
    opt_c = torch.optim.Adam(flat(c1) + flat(c2), lr=ag.hp["lr_critic"], betas=(ag.hp["adam_b1"], ag.hp["adam_b2"]), eps=ag.hp["adam_eps"])
    opt_a = torch.optim.Adam(flat(actor), lr=ag.hp["lr_actor"], betas=(ag.hp["adam_b1"], ag.hp["adam_b2"]), eps=ag.hp["adam_eps"])
    for t in range(5):
        s, a, r, d, s2 = [torch.tensor(x) for x in _batch(ag, t)]
        ag.step()
        eps = torch.tensor(ag.last["eps"])                 # the noise draw is pinned in test_oracle_philox
        with torch.no_grad():
            noise = (ag.hp["policy_noise"] * eps).clamp(-ag.hp["noise_clip"], ag.hp["noise_clip"])
            at = (_tf(ta, s2, 'tanh') + noise).clamp(-1, 1)
            x2 = torch.cat([s2, at], 1)
            y = r + ag.hp["gamma"] * (1 - d) * torch.minimum(_tf(tc1, x2, 'lin'), _tf(tc2, x2, 'lin'))[:, 0]
        x = torch.cat([s, a], 1)
        loss = torch.nn.functional.mse_loss(_tf(c1, x, 'lin')[:, 0], y) + torch.nn.functional.mse_loss(_tf(c2, x, 'lin')[:, 0], y)
        opt_c.zero_grad(); loss.backward(); opt_c.step()
        assert abs(loss.item() - ag.last["critic_loss"]) < 1e-10 * max(1, abs(loss.item()))
        if t % 2 == 0:
            la = -_tf(c1, torch.cat([s, _tf(actor, s, 'tanh')], 1), 'lin').mean()
            opt_a.zero_grad(); la.backward(); opt_a.step()
            assert abs(la.item() - ag.last["actor_loss"]) < 1e-10 * max(1, abs(la.item()))
            with torch.no_grad():
                for tgt, src in ((ta, actor), (tc1, c1), (tc2, c2)):
                    for (Wt, bt), (W, b) in zip(tgt, src):
                        Wt.mul_(1 - ag.hp["tau"]).add_(ag.hp["tau"] * W); bt.mul_(1 - ag.hp["tau"]).add_(ag.hp["tau"] * b)
        else:
            assert ag.last["actor_grads"] is None
    for mine, theirs in ((ag.actor, actor), (ag.critic[0], c1), (ag.critic[1], c2),
                         (ag.t_actor, ta), (ag.t_critic[0], tc1), (ag.t_critic[1], tc2)):
        for (W, b), (tW, tb) in zip(mine, theirs):
            np.testing.assert_allclose(W, tW.detach().numpy(), rtol=1e-9, atol=1e-11)
            np.testing.assert_allclose(b, tb.detach().numpy(), rtol=1e-9, atol=1e-11)


# ---- ordering inside the step ----------------------------------------------------
def test_actor_uses_the_critic_after_its_update():
    for lr_c, expect_equal in ((0.0, True), (1e-2, False)):
        ag = _agent(dict(HP, lr_critic=lr_c))
        s = _batch(ag, 0)[0]
        _, pre = ag.actor_loss_and_grads(s)                # with the critic before its update
        ag.step()
        same = all(np.array_equal(a, b) for x, y in zip(pre, ag.last["actor_grads"]) for a, b in zip(x, y))
        assert same == expect_equal


def test_delayed_steps_leave_actor_and_all_targets_untouched():
    ag = _agent(dict(HP, policy_delay=2))
    snap = lambda: copy.deepcopy((ag.actor, ag.t_actor, ag.t_critic, ag.opt_actor.m, ag.opt_actor.v))
    s0 = snap(); c0 = copy.deepcopy(ag.critic)
    ag.step()                                              # t = 0: everything moves
    s1 = snap(); c1 = copy.deepcopy(ag.critic)
    assert not np.array_equal(s0[0][0][0], s1[0][0][0]) and not np.array_equal(s0[2][0][0][0], s1[2][0][0][0])
    ag.step()                                              # t = 1: critics only
    s2 = snap()
    assert mlp.flatten(s1[0]).tolist() == mlp.flatten(s2[0]).tolist()
    assert mlp.flatten(s1[1]).tolist() == mlp.flatten(s2[1]).tolist()
    for k in range(2):
        assert mlp.flatten(s1[2][k]).tolist() == mlp.flatten(s2[2][k]).tolist()
    assert mlp.flatten(s1[3]).tolist() == mlp.flatten(s2[3]).tolist()
    assert not np.array_equal(c1[0][0][0], ag.critic[0][0][0])
    ag3 = _agent(dict(HP, policy_delay=3))
    moved = []
    for t in range(7):
        before = mlp.flatten(ag3.actor).copy()
        ag3.step()
        moved.append(not np.array_equal(before, mlp.flatten(ag3.actor)))
    assert moved == [True, False, False, True, False, False, True]


def test_targets_start_as_copies_and_polyak_moves_them_towards_online():
    ag = _agent()
    assert np.array_equal(mlp.flatten(ag.actor), mlp.flatten(ag.t_actor))
    assert np.array_equal(mlp.flatten(ag.critic[1]), mlp.flatten(ag.t_critic[1]))
    old_t = mlp.flatten(ag.t_critic[0]).copy()
    ag.step()
    tau = ag.hp["tau"]
    np.testing.assert_allclose(mlp.flatten(ag.t_critic[0]), (1 - tau) * old_t + tau * mlp.flatten(ag.critic[0]), rtol=1e-14, atol=1e-16)


# ---- population independence (Sec. 4.1: replicas are updated independently) -------
def test_agent_in_population_equals_agent_alone_bit_for_bit():
    hps = workloads.hparams(2, P=4)
    def build(hp_list, agents):
        pop = td3.Population(hp_list, 3, 2, [8, 8], 16, 64)
        for j, i in enumerate(agents):
            tr = workloads.transitions(2, i, 50, obs_dim=3, act_dim=2)
            pop.insert(j, **tr)
        pop.update(4)
        return pop
    full = build(hps, range(4))
    for i in (0, 2, 3):
        alone = build([hps[i]], [i])
        for which in td3.WHICH[:12]:
            assert np.array_equal(full.get_params(i, which), alone.get_params(0, which)), (i, which)


def test_empty_buffer_is_an_error_and_short_buffer_is_fine():
    ag = td3.Agent(HP, 3, 2, [4, 4], 8, 16)
    try:
        ag.step()
        assert False
    except RuntimeError:
        pass
    ag.buffer.insert(np.zeros((2, 3)), np.zeros((2, 2)), np.zeros(2), np.zeros(2), np.zeros((2, 3)))
    ag.step()                                              # count < batch: sampling is with replacement
    assert ag.last["idx"].max() < 2


def test_seed_zero_is_derived_from_population_seed_and_index():
    hp = dict(HP, seed=0)
    pop = td3.Population([hp, hp], 3, 2, [4, 4], 4, 8, seed=99)
    assert pop.agents[0].seed == philox.mix64(99, 0) and pop.agents[1].seed == philox.mix64(99, 1)
    assert not np.array_equal(pop.get_params(0, "actor"), pop.get_params(1, "actor"))


# ---- population-method primitives (App. B.1: worst agents replaced by copies of good ones, new hyperparameters) ----
def _small_population(P=3, steps=5):
    hps = workloads.hparams(2, P=P)
    pop = td3.Population(hps, 3, 2, [8, 8], 16, 64)
    for i in range(P):
        pop.insert(i, **workloads.transitions(2, i, 50, obs_dim=3, act_dim=2))
    pop.update(steps)
    return pop, hps


def test_copied_agent_with_the_parents_seed_and_hparams_stays_identical_to_the_parent():
    pop, hps = _small_population()
    before = {w: pop.get_params(2, w).copy() for w in td3.WHICH[:12]}
    pop.copy_agent(0, 2, with_buffer=True)
    for w in td3.WHICH[:12]:
        assert np.array_equal(pop.get_params(0, w), pop.get_params(2, w)), w          # all of the state arrived
        assert np.array_equal(pop.get_params(2, w), before[w]), w                     # the parent is untouched
    assert pop.agents[0].seed == hps[0]["seed"] and pop.agents[0].hp["lr_critic"] == np.float32(hps[0]["lr_critic"])
    pop.set_hparams(0, hps[2])
    pop.update(6)
    for w in td3.WHICH[:12]:
        assert np.array_equal(pop.get_params(0, w), pop.get_params(2, w)), w
    # a deep copy: the child goes its own way once it has its own hyperparameters again
    pop.set_hparams(0, hps[0])
    pop.update(1)
    assert not np.array_equal(pop.get_params(0, "critic1"), pop.get_params(2, "critic1"))


def test_copy_without_buffer_keeps_the_childs_own_transitions():
    pop, _ = _small_population()
    rows = pop.agents[0].buffer.rows.copy()
    pop.copy_agent(0, 1, with_buffer=False)
    assert np.array_equal(pop.agents[0].buffer.rows, rows)
    assert np.array_equal(pop.get_params(0, "v_actor"), pop.get_params(1, "v_actor"))


def test_new_hparams_act_from_the_next_step_and_keep_the_adam_counts_continuous():
    pop, hps = _small_population(P=2, steps=4)          # delay 2: actor updates at t = 0, 2
    ag = pop.agents[0]
    assert ag.actor_updates == 2
    frozen = dict(hps[0], lr_critic=0.0, policy_delay=3)
    pop.set_hparams(0, frozen)
    c_before, a_before = pop.get_params(0, "critic1").copy(), pop.get_params(0, "actor").copy()
    pop.update(2)                                       # t = 4, 5: no multiple of 3
    assert np.array_equal(pop.get_params(0, "critic1"), c_before)      # lr 0: moments move, parameters do not
    assert np.array_equal(pop.get_params(0, "actor"), a_before) and ag.actor_updates == 2
    assert not np.array_equal(pop.get_params(1, "critic1"), pop.get_params(0, "critic1"))
    # t = 6 is an actor step under delay 3; its Adam step is the 3rd, whatever t // delay says.
    # Check against the closed form of one Adam step from the moments before it.
    m0, v0 = pop.get_params(0, "m_actor").copy(), pop.get_params(0, "v_actor").copy()
    pop.update(1)
    assert ag.actor_updates == 3
    g = mlp.flatten(ag.last["actor_grads"])
    b1, b2, eps, lr = ag.hp["adam_b1"], ag.hp["adam_b2"], ag.hp["adam_eps"], ag.hp["lr_actor"]
    m1, v1 = b1 * m0 + (1 - b1) * g, b2 * v0 + (1 - b2) * g * g
    want = a_before - lr * (m1 / (1 - b1 ** 3)) / (np.sqrt(v1 / (1 - b2 ** 3)) + eps)
    np.testing.assert_allclose(pop.get_params(0, "actor"), want, rtol=1e-12, atol=1e-15)


# ---- acting with exploration noise -------------------------------------------------------
def test_exploration_noise_hand_cases():
    ag = _agent()
    obs = np.random.default_rng(3).standard_normal((4000, 3))
    mu = ag.act(obs)
    assert np.array_equal(ag.act(obs, sigma=0.0, step=7), mu)                  # no noise asked for
    a = ag.act(obs, sigma=0.05, step=7)
    assert np.all(np.abs(a) <= 1.0)
    inner = np.abs(mu) < 0.5                                                   # far from the clip: a - mu is the noise itself
    z = (a - mu)[inner] / np.float32(0.05)
    assert abs(z.mean()) < 0.05 and abs(z.std() - 1.0) < 0.03                  # unit normals scaled by sigma
    assert abs(np.mean(z ** 3)) < 0.15 and abs(np.mean(z ** 4) - 3.0) < 0.3    # symmetric, Gaussian kurtosis
    assert np.array_equal(ag.act(obs, sigma=0.05, step=7), a)                  # a function of (seed, step, row, column)
    assert not np.array_equal(ag.act(obs, sigma=0.05, step=8), a)
    assert np.array_equal(ag.act(obs[:100], sigma=0.05, step=7), a[:100])      # row r always gets the same numbers
    big = ag.act(obs, sigma=50.0, step=1)                                      # saturating noise ends on the bounds
    assert np.mean(np.abs(big) == 1.0) > 0.95
    other = _agent(hp=dict(HP, seed=12))
    other.actor = ag.actor
    assert not np.array_equal(other.act(obs, sigma=0.05, step=7), a)           # keyed by the agent's seed
    # independent of the smoothing-noise stream of the update step
    smooth = philox.normals(ag.seed, 4000 * 2, 7, philox.STREAM_SMOOTH).reshape(4000, 2)
    assert abs(np.corrcoef(smooth[inner[:, 0], 0], ((a - mu)[:, 0])[inner[:, 0]])[0, 1]) < 0.06
