"""Helpers for the GPU parity tests: build the HIP population and the oracle on
identical seeded inputs."""
import os

import numpy as np

import paper_2206_08888_amd as pp
import workloads
from oracle import td3 as oracle_td3

NETS = ("actor", "critic1", "critic2")


def ensure_built():
    if not os.path.exists(pp.lib_path()):
        from paper_2206_08888_amd import build
        build.build()
    return pp.load_library()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def make_pair(config_id=0, P=None, capacity=None, fill=None, batch=None, hps=None, agents=None, oracle=True,
              obs_dim=None, act_dim=None):
    """HIP population + oracle population fed with the same hyperparameters and
    transitions.  `agents` selects which population members the oracle holds."""
    cfgd = workloads.CONFIGS[config_id]
    P = cfgd["P"] if P is None else P
    capacity = cfgd["capacity"] if capacity is None else capacity
    fill = capacity if fill is None else fill
    batch = cfgd["batch"] if batch is None else batch
    O = cfgd["obs_dim"] if obs_dim is None else obs_dim
    A = cfgd["act_dim"] if act_dim is None else act_dim
    hps = workloads.hparams(config_id, P) if hps is None else hps
    cfg = pp.make_config(P, O, A, cfgd["hidden"], batch, capacity)
    gpu = pp.Population(cfg, hps)
    agents = list(range(P)) if agents is None else list(agents)
    orc = None
    if oracle:
        orc = oracle_td3.Population([hps[i] for i in agents], O, A, list(cfgd["hidden"]), batch, capacity)
    for i in range(P):
        for tr in workloads.transition_chunks(config_id, i, fill):
            if obs_dim is not None or act_dim is not None:
                raise NotImplementedError
            gpu.insert(i, **tr)
            if oracle and i in agents:
                orc.insert(agents.index(i), **tr)
    return gpu, orc, agents
