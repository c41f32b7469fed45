"""Pins for oracle/td3_shared.py (Sec. 4.2 of the paper: one critic pair for the whole population,
the critic loss averaged over the agents, every policy updated as in single-agent TD3)."""
import copy

import numpy as np
import torch

import workloads
from oracle import mlp, philox, td3, td3_shared
from test_oracle_td3 import _fd_check, _tf, _tnet

HP = dict(workloads.DEFAULT_HP)


def _hps(P, **over):
    rng = np.random.default_rng(17)
    out = []
    for i in range(P):
        hp = dict(HP, seed=101 + i, **over)
        hp["lr_actor"] = float(np.float32(np.exp(rng.uniform(np.log(1e-4), np.log(1e-3)))))
        hp["gamma"] = float(np.float32(rng.uniform(0.9, 0.99)))
        hp["policy_noise"] = float(np.float32(rng.uniform(0.1, 0.3)))
        hp["tau"] = float(np.float32(rng.uniform(0.001, 0.01)))
        out.append(hp)
    return out


def _fill(pop, O, A, fill, data_seed=0):
    for i in range(len(pop.agents)):
        rng = np.random.default_rng(1000 * data_seed + i)
        pop.insert(i, rng.standard_normal((fill, O)), rng.uniform(-1, 1, (fill, A)), rng.standard_normal(fill),
                   (rng.random(fill) < 0.3).astype(np.float32), rng.standard_normal((fill, O)))


def _pop(P=3, O=3, A=2, hidden=(4, 4), B=5, cap=50, fill=40, **over):
    pop = td3_shared.Population(_hps(P, **over), O, A, list(hidden), B, cap)
    _fill(pop, O, A, fill)
    return pop


def test_population_of_one_is_plain_td3_step_for_step():
    hps = _hps(1)
    shared = td3_shared.Population(hps, 3, 2, [4, 4], 5, 50)
    plain = td3.Population(hps, 3, 2, [4, 4], 5, 50)
    _fill(shared, 3, 2, 40); _fill(plain, 3, 2, 40)
    for _ in range(7):
        shared.update(1); plain.update(1)
        for w in td3.WHICH[:12]:
            np.testing.assert_array_equal(shared.get_params(0, w), plain.get_params(0, w))


def test_all_agents_see_one_critic_initialised_from_agent_zero():
    pop = _pop()
    ref = td3.Agent(pop.agents[0].hp, 3, 2, [4, 4], 5, 50)
    for k in range(2):
        for (W, b), (W0, b0) in zip(pop.critic[k], ref.critic[k]):
            np.testing.assert_array_equal(W, W0)
        for ag in pop.agents:
            assert ag.critic[k] is pop.critic[k] and ag.t_critic[k] is pop.t_critic[k]
    for w in ("critic1", "t_critic2", "m_critic1"):
        np.testing.assert_array_equal(pop.get_params(0, w), pop.get_params(2, w))
    assert not np.array_equal(pop.get_params(0, "actor"), pop.get_params(1, "actor"))


def _population_critic_loss(pop, t, ys):
    """(1/P) sum_i (1/B) sum_b sum_k (Q_k - y)^2 written out on the raw arrays."""
    total = 0.0
    for ag, y in zip(pop.agents, ys):
        idx = philox.sample_indices(ag.seed, t, ag.B, ag.buffer.count)
        s, a = (x.astype(np.float64) for x in ag.buffer.gather(idx)[:2])
        x = np.concatenate([s, a], axis=1)
        for k in range(2):
            h = x
            for l, (W, b) in enumerate(pop.critic[k]):
                h = h @ W + b
                if l < 2:
                    h = np.maximum(h, 0.0)
            total += np.mean((h[:, 0] - y) ** 2)
    return total / len(pop.agents)


def test_critic_gradient_is_that_of_the_population_averaged_loss():
    pop = _pop()
    for net in pop.critic:
        for _, b in net:
            b += 0.1
    before = copy.deepcopy(pop.critic)
    pop.step()
    ys = [ag.last["y"] for ag in pop.agents]
    grads = pop.last["critic_grads"]
    after = copy.deepcopy(pop.critic)
    for k in range(2):                                      # back to the weights the gradient was taken at
        for (W, b), (W0, b0) in zip(pop.critic[k], before[k]):
            W[...] = W0; b[...] = b0
    assert abs(_population_critic_loss(pop, 0, ys) - pop.last["critic_loss"]) < 1e-12
    _fd_check(pop.critic, lambda: _population_critic_loss(pop, 0, ys), grads)
    for k in range(2):
        for (W, b), (W1, b1) in zip(pop.critic[k], after[k]):
            W[...] = W1; b[...] = b1


def test_critic_gradient_is_the_mean_of_the_single_agent_gradients():
    pop = _pop(P=4)
    singles = []
    for ag in pop.agents:                                   # each agent alone, plain TD3 pieces, same critic
        lone = td3.Agent(ag.hp, 3, 2, [4, 4], 5, 50)
        lone.buffer, lone.t_actor = copy.deepcopy(ag.buffer), copy.deepcopy(ag.t_actor)
        lone.critic, lone.t_critic = copy.deepcopy(pop.critic), copy.deepcopy(pop.t_critic)
        idx = philox.sample_indices(lone.seed, 0, lone.B, lone.buffer.count)
        s, a, r, d, s2 = (x.astype(np.float64) for x in lone.buffer.gather(idx))
        eps = philox.normals(lone.seed, lone.B * lone.A, 0, philox.STREAM_SMOOTH).reshape(lone.B, lone.A)
        y = lone.bellman_target(r, d, s2, lone.target_action(s2, eps))
        singles.append(lone.critic_loss_and_grads(s, a, y))
    pop.step()
    assert abs(np.mean([l for l, _ in singles]) - pop.last["critic_loss"]) < 1e-13
    for k in range(2):
        mean = mlp.flatten([(np.mean([g[k][l][0] for _, g in singles], axis=0), np.mean([g[k][l][1] for _, g in singles], axis=0))
                            for l in range(3)])
        np.testing.assert_allclose(pop.get_params(0, "g_critic%d" % (k + 1)), mean, rtol=1e-12, atol=1e-15)


def test_actors_move_as_plain_td3_actors_given_the_updated_critic():
    pop = _pop(P=3)
    actors = [copy.deepcopy(ag.actor) for ag in pop.agents]
    pop.step()                                              # t = 0 is a delayed step
    for i, ag in enumerate(pop.agents):
        lone = td3.Agent(ag.hp, 3, 2, [4, 4], 5, 50)
        lone.actor, lone.critic = actors[i], copy.deepcopy(pop.critic)    # the critic AFTER its update
        idx = ag.last["idx"]
        s = ag.buffer.gather(idx)[0].astype(np.float64)
        loss, g = lone.actor_loss_and_grads(s)
        assert abs(loss - ag.last["actor_loss"]) < 1e-13
        np.testing.assert_allclose(mlp.flatten(g), pop.get_params(i, "g_actor"), rtol=1e-12, atol=1e-16)


def test_delay_is_common_and_odd_steps_touch_only_the_critics():
    hps = _hps(2)
    hps[1]["policy_delay"] = 3
    try:
        td3_shared.Population(hps, 3, 2, [4, 4], 5, 50)
        assert False, "mixed delays must be refused"
    except ValueError:
        pass
    pop = _pop(P=2)
    pop.update(1)
    keep = {(i, w): pop.get_params(i, w).copy() for i in range(2) for w in ("actor", "t_actor", "t_critic1", "t_critic2")}
    c1 = pop.get_params(0, "critic1").copy()
    pop.update(1)                                           # t = 1 with delay 2
    for (i, w), v in keep.items():
        np.testing.assert_array_equal(pop.get_params(i, w), v)
    assert not np.array_equal(pop.get_params(0, "critic1"), c1)


def test_three_steps_match_torch_autograd_and_adam():
    P = 3
    pop = _pop(P=P, O=5, A=2, hidden=(16, 16), B=8, cap=200, fill=150)
    hp0 = pop.agents[0].hp
    c1, c2 = _tnet(pop.critic[0]), _tnet(pop.critic[1])
    tc1, tc2 = _tnet(pop.t_critic[0]), _tnet(pop.t_critic[1])
    actors = [_tnet(ag.actor) for ag in pop.agents]
    tactors = [_tnet(ag.t_actor) for ag in pop.agents]
    flat = lambda net: [p for Wb in net for p in Wb]
    opt_c = torch.optim.Adam(flat(c1) + flat(c2), lr=hp0["lr_critic"], betas=(hp0["adam_b1"], hp0["adam_b2"]), eps=hp0["adam_eps"])
    opt_a = [torch.optim.Adam(flat(a), lr=ag.hp["lr_actor"], betas=(ag.hp["adam_b1"], ag.hp["adam_b2"]), eps=ag.hp["adam_eps"])
             for a, ag in zip(actors, pop.agents)]
    for t in range(3):
        data = []
        for ag in pop.agents:
            idx = philox.sample_indices(ag.seed, t, ag.B, ag.buffer.count)
            eps = philox.normals(ag.seed, ag.B * ag.A, t, philox.STREAM_SMOOTH).reshape(ag.B, ag.A)
            data.append([torch.tensor(x.astype(np.float64)) for x in ag.buffer.gather(idx)] + [torch.tensor(eps)])
        pop.step()
        loss = 0.0
        for i, ag in enumerate(pop.agents):
            s, a, r, d, s2, eps = data[i]
            with torch.no_grad():
                noise = (ag.hp["policy_noise"] * eps).clamp(-ag.hp["noise_clip"], ag.hp["noise_clip"])
                at = (_tf(tactors[i], s2, 'tanh') + noise).clamp(-1, 1)
                x2 = torch.cat([s2, at], 1)
                y = r + ag.hp["gamma"] * (1 - d) * torch.minimum(_tf(tc1, x2, 'lin'), _tf(tc2, x2, 'lin'))[:, 0]
            x = torch.cat([s, a], 1)
            loss = loss + (torch.nn.functional.mse_loss(_tf(c1, x, 'lin')[:, 0], y)
                           + torch.nn.functional.mse_loss(_tf(c2, x, 'lin')[:, 0], y)) / P
        opt_c.zero_grad(); loss.backward(); opt_c.step()
        assert abs(loss.item() - pop.last["critic_loss"]) < 1e-10 * max(1, abs(loss.item()))
        if t % 2 == 0:
            for i, ag in enumerate(pop.agents):
                s = data[i][0]
                la = -_tf(c1, torch.cat([s, _tf(actors[i], s, 'tanh')], 1), 'lin').mean()
                opt_a[i].zero_grad(); opt_c.zero_grad(); la.backward(); opt_a[i].step()
                with torch.no_grad():
                    for (Wt, bt), (W, b) in zip(tactors[i], actors[i]):
                        Wt.mul_(1 - ag.hp["tau"]).add_(ag.hp["tau"] * W); bt.mul_(1 - ag.hp["tau"]).add_(ag.hp["tau"] * b)
            with torch.no_grad():
                for tgt, src in ((tc1, c1), (tc2, c2)):
                    for (Wt, bt), (W, b) in zip(tgt, src):
                        Wt.mul_(1 - hp0["tau"]).add_(hp0["tau"] * W); bt.mul_(1 - hp0["tau"]).add_(hp0["tau"] * b)
    pairs = [(pop.critic[0], c1), (pop.critic[1], c2), (pop.t_critic[0], tc1), (pop.t_critic[1], tc2)]
    pairs += [(ag.actor, a) for ag, a in zip(pop.agents, actors)] + [(ag.t_actor, a) for ag, a in zip(pop.agents, tactors)]
    for mine, theirs in pairs:
        for (W, b), (tW, tb) in zip(mine, theirs):
            np.testing.assert_allclose(W, tW.detach().numpy(), rtol=1e-9, atol=1e-11)
            np.testing.assert_allclose(b, tb.detach().numpy(), rtol=1e-9, atol=1e-11)
