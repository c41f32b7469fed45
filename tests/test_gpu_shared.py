"""GPU parity of TD3 with shared critics (Sec. 4.2 of the paper) against oracle/td3_shared.py, through the
C boundary.  Tolerances as for TD3 (test_gpu_parity.py): initial parameters bit-exact; single steps from a common
state element by element (a ReLU unit resolved the other way must be demonstrated as such); free-running steps per
tensor, relative L2 <= 1e-4 after a few steps and <= 1e-3 after 100."""
import numpy as np
import pytest

import paper_2206_08888_amd as pp
import workloads
from gpu_common import check_step_elementwise, check_tensors_all, ensure_built, rel_l2, snapshot
from oracle import td3_shared as oracle_shared

pytestmark = pytest.mark.gpu

ACTOR_SIDE = ("actor", "t_actor")
CRITIC_SIDE = ("critic1", "critic2", "t_critic1", "t_critic2")
MOMS_A = ("m_actor", "v_actor")
MOMS_C = ("m_critic1", "m_critic2", "v_critic1", "v_critic2")


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def make_shared_pair(P=3, capacity=1500, hps=None, oracle=True, config_id=2, obs_dim=17, act_dim=6):
    hps = workloads.hparams(config_id, P) if hps is None else hps      # per-agent lr, tau, noise; one policy delay
    cfg = pp.make_config(P, obs_dim, act_dim, (256, 256), 256, capacity, algo=pp.POP_ALGO_TD3_SHARED)
    gpu = pp.Population(cfg, hps)
    orc = oracle_shared.Population(hps, obs_dim, act_dim, [256, 256], 256, capacity) if oracle else None
    for i in range(P):
        chunks = (workloads.transition_chunks(2, i, capacity) if (obs_dim, act_dim) == (17, 6)
                  else [workloads.transitions(2, i, capacity, obs_dim=obs_dim, act_dim=act_dim, salt=1)])
        for tr in chunks:
            gpu.insert(i, **tr)
            if oracle:
                orc.insert(i, **tr)
    return gpu, orc


def compare(gpu, orc, tol, label, steps=1):
    """After free-running steps: the one critic pair and every policy, as whole networks and tensor by tensor."""
    P = len(orc.agents)
    worst = max(check_tensors_all(gpu, orc, [(0, 0)], CRITIC_SIDE, tol, label, steps=steps),
                check_tensors_all(gpu, orc, [(i, i) for i in range(P)], ACTOR_SIDE, tol, label, steps=steps))
    assert worst <= tol, "%s: worst network rel-L2 %.3e > %.1e" % (label, worst, tol)
    print("%s: worst parameter rel-L2 %.3e (tol %.1e), every tensor within the same tolerance" % (label, worst, tol))


def force(gpu, orc):
    for w in CRITIC_SIDE + MOMS_C:
        gpu.set_params(0, w, orc.get_params(0, w))
    for i in range(len(orc.agents)):
        for w in ACTOR_SIDE + MOMS_A:
            gpu.set_params(i, w, orc.get_params(i, w))


def test_initial_state_one_critic_pair_from_agent_zero():
    gpu, orc = make_shared_pair()
    for i in range(3):
        for w in ACTOR_SIDE + CRITIC_SIDE:
            assert np.array_equal(gpu.get_params(i, w), orc.get_params(i, w).astype(np.float32)), (i, w)
    assert np.array_equal(gpu.get_params(0, "critic2"), gpu.get_params(2, "critic2"))
    assert not np.array_equal(gpu.get_params(0, "actor"), gpu.get_params(1, "actor"))
    gpu.close()


def test_one_step_matches_oracle():
    gpu, orc = make_shared_pair()
    gpu.set_debug(True)
    before = snapshot(orc, range(3))
    gpu.update(1); orc.update(1)
    ties = []
    rep = check_step_elementwise(gpu, orc, [(i, i) for i in range(3)], before, "one step, shared critics", ties=ties)
    print("one step, shared critics: %s; ties %s" % (rep, ties))
    compare(gpu, orc, 1e-4, "one step, shared critics")
    losses = gpu.debug("losses")
    assert abs(losses[0, 0] - orc.last["critic_loss"]) <= 1e-5 * abs(orc.last["critic_loss"])
    assert np.all(losses[:, 0] == losses[0, 0])             # the population's critic loss, reported for every agent
    for i, ag in enumerate(orc.agents):
        assert abs(losses[i, 1] - ag.last["actor_loss"]) <= 1e-5 * max(1.0, abs(ag.last["actor_loss"]))
    assert gpu.step_count() == 1
    gpu.close()


def test_thirty_forced_single_steps_match_oracle():
    gpu, orc = make_shared_pair()
    gpu.set_debug(True)
    pairs = [(i, i) for i in range(3)]
    ties, rep = [], None
    for step in range(30):
        force(gpu, orc)
        before = snapshot(orc, range(3))
        gpu.update(1); orc.update(1)
        rep = check_step_elementwise(gpu, orc, pairs, before, "forced step %d, shared critics" % step, ties=ties, report=rep)
    print("30 forced steps, shared critics: %s; %d network updates behind a ReLU tie: %s" % (rep, len(ties), ties))
    assert len(ties) <= 10
    gpu.close()


@pytest.mark.parametrize("obs_dim,act_dim", [(111, 8), (376, 17)])
def test_wide_shapes_forced_single_steps_match_oracle(obs_dim, act_dim):
    """Shared critics at the Ant and Humanoid shapes: the chains of the wide shapes, one launch per part, the critics'
    weight step with 2 x 4 and 2 x 13 first-layer tile rows."""
    gpu, orc = make_shared_pair(capacity=600, obs_dim=obs_dim, act_dim=act_dim)
    gpu.set_debug(True)
    pairs = [(i, i) for i in range(3)]
    ties, rep = [], None
    for step in range(8):
        force(gpu, orc)
        before = snapshot(orc, range(3))
        gpu.update(1); orc.update(1)
        rep = check_step_elementwise(gpu, orc, pairs, before, "forced step %d, shared critics, obs %d, act %d" % (step, obs_dim, act_dim),
                                     ties=ties, report=rep)
    print("8 forced steps, shared critics at obs %d, act %d: %s; %d network updates behind a ReLU tie: %s" % (obs_dim, act_dim, rep, len(ties), ties))
    assert len(ties) <= 8
    gpu.close()


def test_hundred_steps_match_oracle():
    gpu, orc = make_shared_pair(P=2, hps=workloads.hparams(0, 2), capacity=2000)
    gpu.update(100); orc.update(100)
    compare(gpu, orc, 1e-3, "100 steps, shared critics", steps=100)
    assert gpu.step_count() == 100
    gpu.close()


def test_population_of_one_equals_plain_td3():
    """Same chains, same inputs; the critic's weight step goes through the partial sums and a separate Adam kernel,
    so the last bit may differ (fused multiply-adds are formed per kernel): fp32 rounding level, not bit identity."""
    hps = workloads.hparams(2, 1)
    shared, _ = make_shared_pair(P=1, capacity=1200, hps=hps, oracle=False)
    plain = pp.Population(pp.make_config(1, 17, 6, (256, 256), 256, 1200), hps)
    for tr in workloads.transition_chunks(2, 0, 1200):
        plain.insert(0, **tr)
    shared.update(6); plain.update(6)
    for w in ACTOR_SIDE + CRITIC_SIDE + MOMS_A + MOMS_C:
        e = rel_l2(shared.get_params(0, w), plain.get_params(0, w))
        assert e <= 5e-6, (w, e)
    shared.close(); plain.close()


def test_agents_in_uneven_groups_match_oracle():
    """P = 27: the critic gradient is summed in 20 groups of one or two agents.  With 3.5 million hidden
    pre-activations per critic and step, one of them usually lies within fp32 rounding of zero and is resolved
    differently by the two precisions; the comparison demands that the device's critic gradient then be the oracle's
    with exactly that unit flipped, and holds the step -- the critics, and every policy behind critic 1 -- to the
    ordinary element-wise tolerance against the oracle's arithmetic on that gradient."""
    P = 27
    gpu, orc = make_shared_pair(P=P, capacity=500)
    gpu.set_debug(True)
    pairs = [(i, i) for i in range(P)]
    before = snapshot(orc, range(P))
    gpu.update(1); orc.update(1)
    ties = []
    rep = check_step_elementwise(gpu, orc, pairs, before, "first step at P = %d, shared critics" % P, ties=ties)
    print("first step at P = %d, shared critics: %s; ties %s" % (P, rep, ties))
    force(gpu, orc)
    gpu.update(2); orc.update(2)
    compare(gpu, orc, 1e-4, "two steps from a common state at P = %d, shared critics" % P, steps=2)
    gpu.close()


def test_copy_agent_copies_the_policy_side_only_and_delays_stay_common():
    gpu, _ = make_shared_pair(oracle=False)
    gpu.update(3)
    critic = {w: gpu.get_params(0, w) for w in CRITIC_SIDE + MOMS_C}
    gpu.copy_agent(2, 0, False)
    for w in ACTOR_SIDE + MOMS_A:
        assert np.array_equal(gpu.get_params(2, w), gpu.get_params(0, w)), w
    for w, v in critic.items():
        assert np.array_equal(gpu.get_params(1, w), v), w
    hp = dict(workloads.hparams(2, 3)[1], policy_delay=3)
    with pytest.raises(pp.PopError) as e:
        gpu.set_hparams(1, hp)
    assert e.value.code == pp.POP_EINVAL
    gpu.close()
    mixed = workloads.hparams(2, 3)
    mixed[2]["policy_delay"] = 1
    with pytest.raises(pp.PopError) as e:
        pp.Population(pp.make_config(3, 17, 6, (256, 256), 256, 500, algo=pp.POP_ALGO_TD3_SHARED), mixed)
    assert e.value.code == pp.POP_EINVAL
