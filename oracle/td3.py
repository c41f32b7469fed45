"""Population TD3 update step, one agent at a time (test infrastructure only).

What is computed (Sec. 4.1 of the paper): N replicas of a TD3 agent, each with
its own weights, hyperparameters, seed and replay buffer, each taking the
ordinary single-agent TD3 update (Fujimoto et al. 2018, cited by the paper).
Vectorising over the population only rearranges N independent computations,
so the oracle is the plain definition: a Python loop over agents.

One step t (0-based) of one agent, in order:
  1. draw B replay indices (stream 0) and read the rows (App. A);
  2. target action  a~ = clip(pi'(s2) + clip(sigma*eps, -c, c), -1, 1), eps
     from stream 1, element b*A + j;
  3. y = r + gamma (1 - d) min(Q1'(s2, a~), Q2'(s2, a~)), held constant;
  4. critic loss  (1/B) sum_b [(Q1(s,a) - y)^2 + (Q2(s,a) - y)^2]  (mean over
     the batch, summed over the two critics, no factor 1/2); its gradient by
     hand-derived backprop; Adam on both critics with step count t + 1;
  5. if t mod d == 0: actor loss -(1/B) sum_b Q1(s, pi(s)) through the critic
     just updated in 4 (critic weights get no gradient from it); Adam on the
     actor with its own step count (the number of actor updates taken so far,
     this one included; t/d + 1 while d stays fixed); then Polyak-average all
     three target networks towards the online ones.
Readings taken where the sources the paper cites differ: the actor sees the
critic after its update; all targets move only on delayed steps; step 0 is a
delayed step; sampling is with replacement; ReLU'(0) = 0; `done` is a float
that multiplies the bootstrap term.

Population-method primitives (Sec. 4.2 / App. B.1 of the paper: at the end of an
iteration the worst agents are replaced by copies of good ones and get new
hyperparameters): Population.copy_agent and Population.set_hparams, written as
what the words say -- the copy takes networks, targets, optimiser state and
optionally the buffer; the copy keeps its own seed and hyperparameters until
set_hparams changes them.

Pins: tests/test_oracle_td3.py (finite differences of both losses through the
whole step, torch.autograd float64 cross-check of one full step, hand cases of
the target, step-ordering properties, population independence; a copied agent
given the parent's seed and hyperparameters stays bit-identical to the parent;
hyperparameter changes act from the next step on and leave the Adam counts
continuous).
"""
import numpy as np

from . import mlp, optim, philox, replay

HP_FLOAT_FIELDS = ("lr_actor", "lr_critic", "gamma", "tau", "policy_noise",
                   "noise_clip", "adam_b1", "adam_b2", "adam_eps")


class Agent:
    """All state of one TD3 agent."""

    def __init__(self, hp, obs_dim, act_dim, hidden, batch, capacity):
        self.hp = dict(hp)
        for k in HP_FLOAT_FIELDS:               # the boundary carries these as fp32
            self.hp[k] = float(np.float32(self.hp[k]))
        self.seed = int(hp["seed"])
        self.O, self.A, self.B = obs_dim, act_dim, batch
        a_sizes = [obs_dim] + list(hidden) + [act_dim]
        c_sizes = [obs_dim + act_dim] + list(hidden) + [1]
        self.actor = mlp.init_mlp(self.seed, mlp.NET_ACTOR, a_sizes)
        self.critic = [mlp.init_mlp(self.seed, mlp.NET_CRITIC1, c_sizes),
                       mlp.init_mlp(self.seed, mlp.NET_CRITIC2, c_sizes)]
        self.t_actor = mlp.copy_net(self.actor)
        self.t_critic = [mlp.copy_net(c) for c in self.critic]
        self.opt_actor = optim.AdamState(self.actor)
        self.opt_critic = [optim.AdamState(c) for c in self.critic]
        self.buffer = replay.ReplayBuffer(capacity, obs_dim, act_dim)
        self.t = 0
        self.actor_updates = 0                  # Adam step count of the actor so far
        self.last = {}                          # diagnostics of the last step

    # -- pieces of the step, exposed so tests can pin them one by one ---------
    def target_action(self, s2, eps):
        mu, _ = mlp.forward(self.t_actor, s2, 'tanh')
        sigma, c = self.hp["policy_noise"], self.hp["noise_clip"]
        return np.clip(mu + np.clip(sigma * eps, -c, c), -1.0, 1.0)

    def bellman_target(self, r, d, s2, a_tilde):
        x = np.concatenate([s2, a_tilde], axis=1)
        q1, _ = mlp.forward(self.t_critic[0], x, 'linear')
        q2, _ = mlp.forward(self.t_critic[1], x, 'linear')
        return r + self.hp["gamma"] * (1.0 - d) * np.minimum(q1[:, 0], q2[:, 0])

    def critic_loss_and_grads(self, s, a, y):
        x = np.concatenate([s, a], axis=1)
        B = x.shape[0]
        loss, grads = 0.0, []
        for k in range(2):
            q, cache = mlp.forward(self.critic[k], x, 'linear')
            err = q[:, 0] - y
            loss += np.sum(err * err) / B
            g, _ = mlp.backward(self.critic[k], cache, (2.0 * err / B)[:, None])
            grads.append(g)
        return loss, grads

    def actor_loss_and_grads(self, s):
        B = s.shape[0]
        a_pi, a_cache = mlp.forward(self.actor, s, 'tanh')
        x = np.concatenate([s, a_pi], axis=1)
        q, c_cache = mlp.forward(self.critic[0], x, 'linear')
        loss = -np.sum(q[:, 0]) / B
        _, dx = mlp.backward(self.critic[0], c_cache, np.full((B, 1), -1.0 / B), need_dx=True)
        g, _ = mlp.backward(self.actor, a_cache, dx[:, self.O:])
        return loss, g

    # -- the step -------------------------------------------------------------
    def step(self):
        hp, t = self.hp, self.t
        if self.buffer.count == 0:
            raise RuntimeError("update on an empty replay buffer")
        idx = philox.sample_indices(self.seed, t, self.B, self.buffer.count)
        s, a, r, d, s2 = (x.astype(np.float64) for x in self.buffer.gather(idx))
        eps = philox.normals(self.seed, self.B * self.A, t, philox.STREAM_SMOOTH)
        eps = eps.reshape(self.B, self.A)
        a_tilde = self.target_action(s2, eps)
        y = self.bellman_target(r, d, s2, a_tilde)

        c_loss, c_grads = self.critic_loss_and_grads(s, a, y)
        for k in range(2):
            optim.adam_step(self.critic[k], c_grads[k], self.opt_critic[k], hp["lr_critic"],
                            t + 1, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"])
        self.last = dict(idx=idx, eps=eps, a_tilde=a_tilde, y=y, critic_loss=c_loss,
                         critic_grads=c_grads, actor_grads=None, actor_loss=None)

        delay = int(hp["policy_delay"])
        if t % delay == 0:
            a_loss, a_grads = self.actor_loss_and_grads(s)
            self.actor_updates += 1
            optim.adam_step(self.actor, a_grads, self.opt_actor, hp["lr_actor"],
                            self.actor_updates, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"])
            optim.polyak(self.t_actor, self.actor, hp["tau"])
            for k in range(2):
                optim.polyak(self.t_critic[k], self.critic[k], hp["tau"])
            self.last.update(actor_grads=a_grads, actor_loss=a_loss)
        self.t = t + 1

    def act(self, obs, sigma=0.0, step=0):
        """Actions of the online actor; sigma > 0: with Gaussian exploration noise,
        a = clip(pi(obs) + sigma * eps, -1, 1), eps = unit normal number r*A + j of the
        agent's exploration stream at counter `step` (r = row of obs)."""
        obs = np.asarray(obs, dtype=np.float64)
        y, _ = mlp.forward(self.actor, obs, 'tanh')
        if sigma > 0.0:
            eps = philox.normals(self.seed, obs.shape[0] * self.A, step, philox.STREAM_EXPLORE)
            y = np.clip(y + float(np.float32(sigma)) * eps.reshape(obs.shape[0], self.A), -1.0, 1.0)
        return y


WHICH = ("actor", "critic1", "critic2", "t_actor", "t_critic1", "t_critic2",
         "m_actor", "m_critic1", "m_critic2", "v_actor", "v_critic1", "v_critic2",
         "g_actor", "g_critic1", "g_critic2")


class Population:
    """P independent agents; every call loops over them (Sec. 4.1)."""

    def __init__(self, hparams, obs_dim, act_dim, hidden, batch, capacity, seed=0):
        hps = []
        for i, hp in enumerate(hparams):
            hp = dict(hp)
            if int(hp["seed"]) == 0:
                hp["seed"] = philox.mix64(seed, i)
            hps.append(hp)
        self.agents = [Agent(hp, obs_dim, act_dim, hidden, batch, capacity) for hp in hps]

    def insert(self, agent, obs, act, rew, done, next_obs):
        self.agents[agent].buffer.insert(obs, act, rew, done, next_obs)

    def update(self, n_steps):
        for ag in self.agents:
            for _ in range(n_steps):
                ag.step()

    def act(self, obs, sigma=None, step=0):
        return np.stack([ag.act(obs[i], 0.0 if sigma is None else sigma[i], step)
                         for i, ag in enumerate(self.agents)])

    def copy_agent(self, dst, src, with_buffer):
        """Agent dst becomes a copy of agent src: online and target networks, Adam moments
        and the actor's Adam count; with_buffer: also the replay buffer (contents, cursor,
        fill level).  dst keeps its own seed and hyperparameters."""
        import copy
        a, b = self.agents[src], self.agents[dst]
        b.actor, b.critic = copy.deepcopy(a.actor), copy.deepcopy(a.critic)
        b.t_actor, b.t_critic = copy.deepcopy(a.t_actor), copy.deepcopy(a.t_critic)
        b.opt_actor, b.opt_critic = copy.deepcopy(a.opt_actor), copy.deepcopy(a.opt_critic)
        b.actor_updates = a.actor_updates
        if with_buffer:
            b.buffer = copy.deepcopy(a.buffer)

    def set_hparams(self, agent, hp):
        """New hyperparameters (and seed) for one agent from its next step on."""
        ag = self.agents[agent]
        ag.hp = dict(hp)
        for k in HP_FLOAT_FIELDS:
            ag.hp[k] = float(np.float32(ag.hp[k]))
        ag.seed = int(hp["seed"])

    def get_params(self, agent, which):
        ag = self.agents[agent]
        table = {
            "actor": ag.actor, "critic1": ag.critic[0], "critic2": ag.critic[1],
            "t_actor": ag.t_actor, "t_critic1": ag.t_critic[0], "t_critic2": ag.t_critic[1],
            "m_actor": ag.opt_actor.m, "m_critic1": ag.opt_critic[0].m, "m_critic2": ag.opt_critic[1].m,
            "v_actor": ag.opt_actor.v, "v_critic1": ag.opt_critic[0].v, "v_critic2": ag.opt_critic[1].v,
            "g_actor": ag.last.get("actor_grads"),
            "g_critic1": ag.last["critic_grads"][0] if ag.last else None,
            "g_critic2": ag.last["critic_grads"][1] if ag.last else None,
        }
        return mlp.flatten(table[which])
