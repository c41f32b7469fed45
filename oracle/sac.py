"""Population SAC update step, one agent at a time (test infrastructure only).

What is computed (Sec. 4.1 of the paper): N replicas of a Soft Actor-Critic agent
(Haarnoja et al. 2018, "Soft actor-critic algorithms and applications", cited by the
paper, with the learned temperature), each with its own weights, hyperparameters, seed
and replay buffer; the same plain definition as for TD3: a Python loop over agents.

The policy is a tanh-squashed diagonal Gaussian: the actor MLP has 2A outputs,
(mu, log_std) = split(actor(s)); log_std is clamped to [-20, 2] (no gradient outside);
u = mu + exp(log_std) eps, eps ~ N(0, I); a = tanh(u);
    log pi(a|s) = sum_j [ -eps_j^2/2 - log_std_j - ln(2 pi)/2 ] - sum_j ln(1 - tanh(u_j)^2),
the last term evaluated as 2 (ln 2 - u - softplus(-2u)).

One step t (0-based) of one agent, in order (alpha = exp(log_alpha) as it stands at the
start of the step, held constant in 2-4):
  1. draw B replay indices (stream 0) and read the rows;
  2. a' ~ pi(.|s') from the ONLINE actor (there is no target actor), eps from stream 3;
     y = r + gamma (1 - d) (min_k Q'_k(s', a') - alpha log pi(a'|s')), held constant;
  3. critic loss (1/B) sum_b [(Q1(s,a) - y)^2 + (Q2(s,a) - y)^2]; Adam on both critics,
     step count t + 1;
  4. a ~ pi(.|s), eps from stream 2; actor loss (1/B) sum_b [alpha log pi(a|s) -
     min_k Q_k(s, a)] through the critics just updated in 3 (they get no gradient from
     it; per sample the gradient flows through the smaller critic, the first on ties);
     Adam on the actor, step count t + 1;
  5. temperature loss -(alpha / B) sum_b (log pi(a|s) + target_entropy) as a function of
     log_alpha with log pi from 4 held constant, i.e. d/dlog_alpha = -alpha mean(log pi +
     target_entropy); one Adam step on log_alpha with lr_alpha, step count t + 1;
  6. Polyak-average the two target critics towards the online ones.
Readings taken where SAC implementations differ (the paper names the algorithm and its
"standard hyperparametrization", not these details): everything is updated every step;
the actor sees the critics after their update; the temperature loss carries alpha (not
log_alpha) as the multiplier; hard clamp of log_std; rewards are used as stored (a
reward scale is applied by whoever fills the buffer).

Pins: tests/test_oracle_sac.py (log pi against scipy's normal density and the change of
variables written out; finite differences of the actor and critic losses through the
whole sampled computation; torch.autograd float64 cross-check of full steps including
the temperature; hand cases of the target and of the temperature update; clamp has no
gradient; step-ordering properties).
"""
import numpy as np

from . import mlp, optim, philox, replay

HP_FLOAT_FIELDS = ("lr_actor", "lr_critic", "gamma", "tau", "adam_b1", "adam_b2", "adam_eps",
                   "lr_alpha", "target_entropy", "init_log_alpha")
LOG_STD_MIN, LOG_STD_MAX = -20.0, 2.0
NET_ACTOR = mlp.NET_ACTOR


def softplus(x):
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def sample_policy(actor, s, eps):
    """(a, log pi(a|s), cache) for the tanh-Gaussian policy with noise eps [B, A]."""
    out, cache = mlp.forward(actor, s, 'linear')
    A = eps.shape[1]
    mu, ls_raw = out[:, :A], out[:, A:]
    ls = np.clip(ls_raw, LOG_STD_MIN, LOG_STD_MAX)
    std = np.exp(ls)
    u = mu + std * eps
    a = np.tanh(u)
    logp = np.sum(-0.5 * eps * eps - ls - 0.5 * np.log(2.0 * np.pi), axis=1) \
        - np.sum(2.0 * (np.log(2.0) - u - softplus(-2.0 * u)), axis=1)
    inside = (ls_raw >= LOG_STD_MIN) & (ls_raw <= LOG_STD_MAX)
    return a, logp, (cache, a, std, eps, inside)


def policy_backward(actor, pcache, d_a, d_logp):
    """Gradient of the actor parameters given dL/da [B, A] and dL/dlog pi [B].

    u = mu + std eps, a = tanh u:  da/du = 1 - a^2;  d(log pi)/du = 2 a  (the Gaussian part
    does not depend on u once eps is fixed; d/du[-ln(1 - tanh^2 u)] = 2 tanh u);
    d(log pi)/d(log_std) = -1 directly, plus the path through u: du/dlog_std = std eps.
    The clamp passes no gradient where log_std was outside its range."""
    cache, a, std, eps, inside = pcache
    d_u = d_a * (1.0 - a * a) + d_logp[:, None] * 2.0 * a
    d_mu = d_u
    d_ls = (d_u * std * eps - d_logp[:, None]) * inside
    grads, _ = mlp.backward(actor, cache, np.concatenate([d_mu, d_ls], axis=1))
    return grads


class Agent:
    """All state of one SAC agent."""

    def __init__(self, hp, obs_dim, act_dim, hidden, batch, capacity):
        self.hp = dict(hp)
        for k in HP_FLOAT_FIELDS:               # the boundary carries these as fp32
            self.hp[k] = float(np.float32(self.hp[k]))
        self.seed = int(hp["seed"])
        self.O, self.A, self.B = obs_dim, act_dim, batch
        a_sizes = [obs_dim] + list(hidden) + [2 * act_dim]
        c_sizes = [obs_dim + act_dim] + list(hidden) + [1]
        self.actor = mlp.init_mlp(self.seed, mlp.NET_ACTOR, a_sizes)
        self.critic = [mlp.init_mlp(self.seed, mlp.NET_CRITIC1, c_sizes),
                       mlp.init_mlp(self.seed, mlp.NET_CRITIC2, c_sizes)]
        self.t_critic = [mlp.copy_net(c) for c in self.critic]
        self.opt_actor = optim.AdamState(self.actor)
        self.opt_critic = [optim.AdamState(c) for c in self.critic]
        self.log_alpha = np.array([self.hp["init_log_alpha"]], dtype=np.float64)
        self.opt_alpha = optim.AdamState([(self.log_alpha, np.zeros(0))])
        self.buffer = replay.ReplayBuffer(capacity, obs_dim, act_dim)
        self.t = 0
        self.last = {}

    # -- pieces of the step, exposed so tests can pin them one by one ---------
    def bellman_target(self, r, d, s2, eps2, alpha):
        a2, logp2, _ = sample_policy(self.actor, s2, eps2)
        x = np.concatenate([s2, a2], axis=1)
        q1, _ = mlp.forward(self.t_critic[0], x, 'linear')
        q2, _ = mlp.forward(self.t_critic[1], x, 'linear')
        return r + self.hp["gamma"] * (1.0 - d) * (np.minimum(q1[:, 0], q2[:, 0]) - alpha * logp2)

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

    def actor_loss_and_grads(self, s, eps, alpha):
        """(loss, grads, log pi) of (1/B) sum [alpha log pi(a|s) - min_k Q_k(s, a)]."""
        B = s.shape[0]
        a, logp, pcache = sample_policy(self.actor, s, eps)
        x = np.concatenate([s, a], axis=1)
        q, caches = [], []
        for k in range(2):
            qk, ck = mlp.forward(self.critic[k], x, 'linear')
            q.append(qk[:, 0]); caches.append(ck)
        first = q[0] <= q[1]                      # ties go to the first critic
        loss = np.sum(alpha * logp - np.where(first, q[0], q[1])) / B
        d_a = np.zeros_like(a)
        for k, sel in ((0, first), (1, ~first)):
            _, dx = mlp.backward(self.critic[k], caches[k], (-1.0 / B * sel)[:, None], need_dx=True)
            d_a += dx[:, self.O:]
        grads = policy_backward(self.actor, pcache, d_a, np.full(B, alpha / B))
        return loss, grads, logp

    # -- the step -------------------------------------------------------------
    def step(self):
        hp, t = self.hp, self.t
        if self.buffer.count == 0:
            raise RuntimeError("update on an empty replay buffer")
        idx = philox.sample_indices(self.seed, t, self.B, self.buffer.count)
        s, a, r, d, s2 = (x.astype(np.float64) for x in self.buffer.gather(idx))
        eps1 = philox.normals(self.seed, self.B * self.A, t, philox.STREAM_SAC_S).reshape(self.B, self.A)
        eps2 = philox.normals(self.seed, self.B * self.A, t, philox.STREAM_SAC_S2).reshape(self.B, self.A)
        alpha = float(np.exp(self.log_alpha[0]))
        y = self.bellman_target(r, d, s2, eps2, alpha)

        c_loss, c_grads = self.critic_loss_and_grads(s, a, y)
        for k in range(2):
            optim.adam_step(self.critic[k], c_grads[k], self.opt_critic[k], hp["lr_critic"],
                            t + 1, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"])

        a_loss, a_grads, logp = self.actor_loss_and_grads(s, eps1, alpha)
        optim.adam_step(self.actor, a_grads, self.opt_actor, hp["lr_actor"],
                        t + 1, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"])

        g_alpha = -alpha * np.mean(logp + hp["target_entropy"])
        optim.adam_step([(self.log_alpha, np.zeros(0))], [(np.array([g_alpha]), np.zeros(0))], self.opt_alpha,
                        hp["lr_alpha"], t + 1, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"])

        for k in range(2):
            optim.polyak(self.t_critic[k], self.critic[k], hp["tau"])
        self.last = dict(idx=idx, eps1=eps1, eps2=eps2, y=y, alpha=alpha, critic_loss=c_loss, critic_grads=c_grads,
                         actor_loss=a_loss, actor_grads=a_grads, logp=logp, alpha_grad=g_alpha)
        self.t = t + 1

    def act(self, obs, deterministic=True, step=0):
        """Mean action tanh(mu); or a sample with eps from the exploration stream at counter `step`."""
        obs = np.asarray(obs, dtype=np.float64)
        out, _ = mlp.forward(self.actor, obs, 'linear')
        mu, ls = out[:, :self.A], np.clip(out[:, self.A:], LOG_STD_MIN, LOG_STD_MAX)
        if deterministic:
            return np.tanh(mu)
        eps = philox.normals(self.seed, obs.shape[0] * self.A, step, philox.STREAM_EXPLORE)
        return np.tanh(mu + np.exp(ls) * eps.reshape(obs.shape[0], self.A))


WHICH = ("actor", "critic1", "critic2", "t_critic1", "t_critic2",
         "m_actor", "m_critic1", "m_critic2", "v_actor", "v_critic1", "v_critic2",
         "log_alpha", "m_log_alpha", "v_log_alpha", "g_actor", "g_critic1", "g_critic2")


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

    def act(self, obs):
        return np.stack([ag.act(obs[i]) for i, ag in enumerate(self.agents)])

    def get_params(self, agent, which):
        ag = self.agents[agent]
        if which in ("log_alpha", "m_log_alpha", "v_log_alpha"):
            return {"log_alpha": ag.log_alpha, "m_log_alpha": ag.opt_alpha.m[0][0],
                    "v_log_alpha": ag.opt_alpha.v[0][0]}[which].copy()
        table = {
            "actor": ag.actor, "critic1": ag.critic[0], "critic2": ag.critic[1],
            "t_critic1": ag.t_critic[0], "t_critic2": ag.t_critic[1],
            "m_actor": ag.opt_actor.m, "m_critic1": ag.opt_critic[0].m, "m_critic2": ag.opt_critic[1].m,
            "v_actor": ag.opt_actor.v, "v_critic1": ag.opt_critic[0].v, "v_critic2": ag.opt_critic[1].v,
            "g_actor": ag.last.get("actor_grads"),
            "g_critic1": ag.last["critic_grads"][0] if ag.last else None,
            "g_critic2": ag.last["critic_grads"][1] if ag.last else None,
        }
        return mlp.flatten(table[which])
