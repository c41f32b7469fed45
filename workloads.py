"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only *describes workloads and draws input data*: population sizes,
shapes, per-agent hyperparameter values and replay transitions.  It contains
none of the method's arithmetic (no networks, no losses, no optimiser, no
replay sampling), so that the CPU oracle and the HIP library can both be fed
from it without sharing code.

The transitions stand in for the paper's benchmark data (Sec. 4.1: generated
training batches shaped like MuJoCo Gym HalfCheetah-v2, obs 17 / act 6, and
Humanoid-v2, obs 376 / act 17); nothing here is recorded environment data.
"""
import numpy as np

# shapes of the continuous-control workloads of Sec. 4.1
HALFCHEETAH = dict(obs_dim=17, act_dim=6)
HUMANOID = dict(obs_dim=376, act_dim=17)

CONFIGS = {
    # 0: small parity case
    0: dict(algo="td3", P=2, hidden=(256, 256), batch=256, capacity=10_000, steps=1,
            sweep=(), **HALFCHEETAH),
    # 1: metric case, P = 10
    1: dict(algo="td3", P=10, hidden=(256, 256), batch=256, capacity=1_000_000, steps=1000,
            sweep=("lr",), **HALFCHEETAH),
    # 2: metric case, P = 80 hyperparameter sweep
    2: dict(algo="td3", P=80, hidden=(256, 256), batch=256, capacity=200_000, steps=1000,
            sweep=("lr", "tau", "policy_noise"), **HALFCHEETAH),
    # 3: SAC variant
    3: dict(algo="sac", P=32, hidden=(256, 256), batch=256, capacity=500_000, steps=500,
            sweep=(), **HUMANOID),
    # 5: SAC at the shapes the paper itself measures SAC on (Sec. 4.1: HalfCheetah-v2), population of config 3
    5: dict(algo="sac", P=32, hidden=(256, 256), batch=256, capacity=200_000, steps=500,
            sweep=("lr", "tau"), **HALFCHEETAH),
    # 6: TD3 with shared critics (Sec. 4.2 of the paper; its runtime figure varies the population size), at the
    #    population and shapes of config 2; one policy delay for all agents
    6: dict(algo="td3_shared", P=80, hidden=(256, 256), batch=256, capacity=200_000, steps=1000,
            sweep=("lr", "tau", "policy_noise"), **HALFCHEETAH),
    # 4: saturation case, P up to 256
    4: dict(algo="td3", P=256, hidden=(256, 256), batch=256, capacity=50_000, steps=200,
            sweep=("lr", "tau", "policy_noise"), **HALFCHEETAH),
}

DEFAULT_HP = dict(seed=0, lr_actor=3e-4, lr_critic=3e-4, gamma=0.99, tau=0.005,
                  policy_noise=0.2, noise_clip=0.5, policy_delay=2,
                  adam_b1=0.9, adam_b2=0.999, adam_eps=1e-8,
                  lr_alpha=3e-4, target_entropy=0.0, init_log_alpha=0.0)

HP_SEED = 220608888
DATA_SEED = 8888


def hparams(config_id, P=None):
    """Per-agent hyperparameters of a config, as a list of plain dicts.

    seed_i = 1 + i + 1000*config; the swept fields are drawn once on the host:
    lr log-uniform in [1e-4, 1e-3] (one value for actor and critic), tau
    uniform in [0.001, 0.01], policy noise uniform in [0.1, 0.3].  Float
    fields are rounded to fp32, the precision the C boundary carries."""
    cfg = CONFIGS[config_id]
    P = cfg["P"] if P is None else P
    rng = np.random.Generator(np.random.Philox(key=HP_SEED + config_id))
    out = []
    for i in range(P):
        hp = dict(DEFAULT_HP)
        hp["seed"] = 1 + i + 1000 * config_id
        # always draw all three so that agent i's values do not depend on `sweep`
        lr = float(np.exp(rng.uniform(np.log(1e-4), np.log(1e-3))))
        tau = float(rng.uniform(0.001, 0.01))
        sigma = float(rng.uniform(0.1, 0.3))
        if "lr" in cfg["sweep"]:
            hp["lr_actor"] = hp["lr_critic"] = lr
        if "tau" in cfg["sweep"]:
            hp["tau"] = tau
        if "policy_noise" in cfg["sweep"]:
            hp["policy_noise"] = sigma
        if cfg["algo"] == "sac":
            hp["target_entropy"] = -float(cfg["act_dim"])
        for k, v in hp.items():
            if isinstance(v, float):
                hp[k] = float(np.float32(v))
        out.append(hp)
    return out


def transitions(config_id, agent, n, obs_dim=None, act_dim=None, salt=0):
    """n synthetic transitions for one agent as fp32 arrays.

    obs, next_obs ~ N(0,1) per element, act ~ U[-1,1], reward ~ N(0,1),
    done ~ Bernoulli(0.01) stored as 0/1.  The stream depends only on
    (config, agent, salt), never on P."""
    cfg = CONFIGS[config_id]
    O = cfg["obs_dim"] if obs_dim is None else obs_dim
    A = cfg["act_dim"] if act_dim is None else act_dim
    key = DATA_SEED + 1000 * config_id + agent + 1_000_000 * salt
    rng = np.random.Generator(np.random.Philox(key=key))
    return dict(
        obs=rng.standard_normal((n, O), dtype=np.float32),
        act=rng.uniform(-1.0, 1.0, (n, A)).astype(np.float32),
        rew=rng.standard_normal(n, dtype=np.float32),
        done=(rng.random(n) < 0.01).astype(np.float32),
        next_obs=rng.standard_normal((n, O), dtype=np.float32),
    )


def transition_chunks(config_id, agent, n, chunk=250_000):
    """Same distributions, generated piecewise for large buffers; chunk c uses
    salt c + 1, so a test can regenerate any agent's buffer on its own."""
    off, c = 0, 1
    while off < n:
        m = min(chunk, n - off)
        yield transitions(config_id, agent, m, salt=c)
        off += m
        c += 1
