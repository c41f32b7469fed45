"""TD3 population with shared critics (test infrastructure only).

What is computed (Sec. 4.2 of the paper, "Training Agents Sharing Parameters"):
every agent has its own policy (and target policy), the two critics and their
targets exist once.  The paper's variant of the scheme of CEM-RL / DvD / QD-PG:
within one update step every agent's batch goes through that agent's policy
networks, all agents in parallel, and the critic loss is the average over the
population; given the critics, each policy takes the single-agent TD3 update.

One step t (0-based), population of P agents:
  1. every agent i draws its batch (its own index stream and buffer) and forms
       a~_i = clip(pi'_i(s2_i) + clip(sigma_i eps_i, -c_i, c_i), -1, 1)
       y_i  = r_i + gamma_i (1 - d_i) min_k Q'_k(s2_i, a~_i)          (shared target critics)
  2. critic loss  L = (1/P) sum_i (1/B) sum_b sum_k (Q_k(s_ib, a_ib) - y_ib)^2 ;
     ONE Adam step on each shared critic with step count t + 1;
  3. if t mod d == 0 (one delay for the whole population): every agent takes the
     TD3 actor step  -(1/B) sum_b Q_1(s_ib, pi_i(s_ib))  through the critic updated
     in 2, its own Adam step, Polyak on its own target policy with its own tau;
     then Polyak on the two shared target critics.
Readings (the paper gives the scheme in one sentence): every agent samples its
own batch, so a step contracts over P*B rows; the shared critic takes its learning
rate, Adam constants, tau and its initial weights (seed) from agent 0's
hyperparameters; gamma and the smoothing noise stay per agent; the policy delay
must be common to all agents.

The single-agent pieces (target action, Bellman target, the two losses and their
hand-derived gradients) are td3.Agent's, applied to the shared networks.

Pins: tests/test_oracle_td3_shared.py (a population of one equals the plain TD3
oracle step for step; finite differences of the population-averaged critic loss;
the critic gradient equals the mean of the gradients the plain oracle computes for
each agent alone on the same critic; actors move exactly as plain TD3 actors would
given that critic; a float64 torch.autograd cross-check of one whole step).
"""
import numpy as np

from . import mlp, optim, philox, td3


class Population:
    def __init__(self, hparams, obs_dim, act_dim, hidden, batch, capacity, seed=0):
        hps = []
        for i, hp in enumerate(hparams):
            hp = dict(hp)
            if int(hp["seed"]) == 0:
                hp["seed"] = philox.mix64(seed, i)
            hps.append(hp)
        delays = {int(hp["policy_delay"]) for hp in hps}
        if len(delays) != 1:
            raise ValueError("shared critics need one policy delay for the whole population")
        self.agents = [td3.Agent(hp, obs_dim, act_dim, hidden, batch, capacity) for hp in hps]
        first = self.agents[0]
        self.critic, self.t_critic, self.opt_critic = first.critic, first.t_critic, first.opt_critic
        for ag in self.agents:                  # every agent sees the same critic objects
            ag.critic, ag.t_critic, ag.opt_critic = self.critic, self.t_critic, self.opt_critic
        self.t = 0
        self.last = {}

    def insert(self, agent, obs, act, rew, done, next_obs):
        self.agents[agent].buffer.insert(obs, act, rew, done, next_obs)

    def step(self):
        t, P = self.t, len(self.agents)
        hp0 = self.agents[0].hp
        batches, c_loss = [], 0.0
        c_grads = [[(np.zeros_like(W), np.zeros_like(b)) for W, b in net] for net in self.critic]
        for ag in self.agents:
            if ag.buffer.count == 0:
                raise RuntimeError("update on an empty replay buffer")
            idx = philox.sample_indices(ag.seed, t, ag.B, ag.buffer.count)
            s, a, r, d, s2 = (x.astype(np.float64) for x in ag.buffer.gather(idx))
            eps = philox.normals(ag.seed, ag.B * ag.A, t, philox.STREAM_SMOOTH).reshape(ag.B, ag.A)
            y = ag.bellman_target(r, d, s2, ag.target_action(s2, eps))
            loss_i, grads_i = ag.critic_loss_and_grads(s, a, y)
            c_loss += loss_i / P
            for k in range(2):
                for l, (gW, gb) in enumerate(grads_i[k]):
                    c_grads[k][l][0][...] += gW / P
                    c_grads[k][l][1][...] += gb / P
            batches.append(s)
            ag.last = dict(idx=idx, y=y, actor_grads=None, actor_loss=None)
        for k in range(2):
            optim.adam_step(self.critic[k], c_grads[k], self.opt_critic[k], hp0["lr_critic"],
                            t + 1, hp0["adam_b1"], hp0["adam_b2"], hp0["adam_eps"])
        self.last = dict(critic_loss=c_loss, critic_grads=c_grads)

        if t % int(hp0["policy_delay"]) == 0:
            for ag, s in zip(self.agents, batches):
                a_loss, a_grads = ag.actor_loss_and_grads(s)
                ag.actor_updates += 1
                optim.adam_step(ag.actor, a_grads, ag.opt_actor, ag.hp["lr_actor"], ag.actor_updates,
                                ag.hp["adam_b1"], ag.hp["adam_b2"], ag.hp["adam_eps"])
                optim.polyak(ag.t_actor, ag.actor, ag.hp["tau"])
                ag.last.update(actor_grads=a_grads, actor_loss=a_loss)
            for k in range(2):
                optim.polyak(self.t_critic[k], self.critic[k], hp0["tau"])
        self.t = t + 1
        for ag in self.agents:
            ag.t = self.t

    def update(self, n_steps):
        for _ in range(n_steps):
            self.step()

    def act(self, obs, sigma=None, step=0):
        return np.stack([ag.act(obs[i], 0.0 if sigma is None else sigma[i], step)
                         for i, ag in enumerate(self.agents)])

    def get_params(self, agent, which):
        """Critic tensors are the shared ones whatever `agent` says."""
        ag = self.agents[agent]
        table = {
            "actor": ag.actor, "critic1": self.critic[0], "critic2": self.critic[1],
            "t_actor": ag.t_actor, "t_critic1": self.t_critic[0], "t_critic2": self.t_critic[1],
            "m_actor": ag.opt_actor.m, "m_critic1": self.opt_critic[0].m, "m_critic2": self.opt_critic[1].m,
            "v_actor": ag.opt_actor.v, "v_critic1": self.opt_critic[0].v, "v_critic2": self.opt_critic[1].v,
            "g_actor": ag.last.get("actor_grads"),
            "g_critic1": self.last["critic_grads"][0] if self.last else None,
            "g_critic2": self.last["critic_grads"][1] if self.last else None,
        }
        return mlp.flatten(table[which])
