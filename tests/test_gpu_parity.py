"""GPU parity: the HIP library against the CPU oracle on identical seeded inputs,
through the C boundary.  Tolerances (fp32 path against the fp64 oracle):
  * replay indices and gathered rows: bit-exact (integer and copy work);
  * initial parameters: bit-exact (one fp32 rounding on both sides);
  * single steps from a common state: every tensor (W1, b1, W2, b2, W3, b3) of every network element by
    element -- gradients within 1e-6 of the tensor's largest entry and 1e-5 relative L2, parameters, targets and
    Adam moments within the tolerance parity_checks.py derives from the Adam update (1e-4 of max(|theta|, lr) on
    well-determined entries), entries with an exactly zero gradient unchanged bit for bit;
  * several free steps: per tensor, relative L2 <= 1e-4 after a few steps and <= 1e-3 after 100 steps (the
    relative L2 of the whole network is asserted as well);
  * a hidden unit within fp32 rounding of its ReLU kink may be resolved differently by the two precisions: such a
    step is accepted only when the device's gradient is reproduced by the oracle's with exactly those units
    flipped (relu_ties.py), and is then compared as strictly as any other."""
import numpy as np
import pytest

import paper_2206_08888_amd as pp
import workloads
from gpu_common import (MOM_M, MOM_V, NETS, PARAMS6, STATE12, check_step_elementwise, check_tensors_all, describe_free_run,
                        ensure_built, force_state, free_run_tie_aware, make_pair, rel_l2, snapshot)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def _compare_state(gpu, orc, agents, tol, label, steps=1):
    """Parameters and targets of every network after `steps` free steps: relative L2 of the whole network and of
    each of its tensors."""
    pairs = [(i, j) for j, i in enumerate(agents)]
    worst = check_tensors_all(gpu, orc, pairs, PARAMS6, tol, label, steps=steps)
    assert worst <= tol, "%s: worst network rel-L2 %.3e > %.1e" % (label, worst, tol)
    print("%s: worst parameter rel-L2 %.3e (tol %.1e), every tensor within the same tolerance" % (label, worst, tol))
    return worst


def test_initial_parameters_are_bit_exact():
    gpu, orc, agents = make_pair(0, capacity=256, fill=256)
    for i in agents:
        for which in ("actor", "critic1", "critic2", "t_actor", "t_critic1", "t_critic2"):
            a = gpu.get_params(i, which)
            b = orc.get_params(i, which).astype(np.float32)
            assert np.array_equal(a, b), (i, which, np.abs(a - b).max())
        for which in ("m_actor", "v_critic2"):
            assert not gpu.get_params(i, which).any()
    gpu.close()


def test_indices_and_gathered_rows_are_bit_exact_over_steps():
    gpu, orc, agents = make_pair(0)
    for step in range(3):
        gpu.update(1)
        orc.update(1)
        idx = gpu.debug("indices")
        rows = gpu.debug("batch")
        for i in agents:
            ag = orc.agents[i]
            assert np.array_equal(idx[i].astype(np.int64), ag.last["idx"]), (step, i)
            assert np.array_equal(rows[i], ag.buffer.rows[ag.last["idx"]]), (step, i)
    gpu.close()


def test_one_step_matches_oracle():
    gpu, orc, agents = make_pair(0)
    gpu.set_debug(1)
    before = snapshot(orc, agents)
    gpu.update(1)
    orc.update(1)
    at = gpu.debug("target_action"); y = gpu.debug("target_y"); losses = gpu.debug("losses")
    for i in agents:
        ag = orc.agents[i]
        assert np.abs(at[i] - ag.last["a_tilde"]).max() <= 2e-6
        assert np.abs(y[i] - ag.last["y"]).max() <= 1e-5 * np.abs(ag.last["y"]).max()
        assert abs(losses[i, 0] - ag.last["critic_loss"]) <= 1e-5 * abs(ag.last["critic_loss"])
        assert abs(losses[i, 1] - ag.last["actor_loss"]) <= 1e-5 * max(1.0, abs(ag.last["actor_loss"]))
        for net in NETS:                                  # network-level figures as before, now beside the element-wise ones
            assert rel_l2(gpu.get_params(i, "g_" + net), orc.get_params(i, "g_" + net)) <= 1e-5
            for mom in ("m_", "v_"):
                assert rel_l2(gpu.get_params(i, mom + net), orc.get_params(i, mom + net)) <= 2e-5
    ties = []
    rep = check_step_elementwise(gpu, orc, [(i, i) for i in agents], before, "config 0, 1 step", ties=ties)
    print("config 0, 1 step: %s; ties %s" % (rep, ties))
    assert rep.masked <= 0.01 * rep.entries
    _compare_state(gpu, orc, agents, 1e-4, "config 0, 1 step")
    gpu.close()


def test_two_steps_cover_the_critic_only_branch():
    gpu, orc, agents = make_pair(0)
    gpu.update(1); orc.update(1)
    snap = {(i, w): gpu.get_params(i, w) for i in agents for w in ("actor", "t_actor", "t_critic1", "t_critic2", "m_actor")}
    gpu.update(1); orc.update(1)
    for (i, w), before in snap.items():          # delayed step: actor and targets bit-unchanged
        assert np.array_equal(before, gpu.get_params(i, w)), (i, w)
    _compare_state(gpu, orc, agents, 1e-4, "config 0, 2 steps", steps=2)
    gpu.close()


def test_hundred_steps_match_oracle():
    """100 free steps in one call: relative L2 <= 1e-3 per network.  The same run taken one step at a time shows
    where the two precisions part: tight agreement (1e-5, per tensor) until a ReLU tie, which is demonstrated."""
    gpu, orc, agents = make_pair(0)
    gpu.update(100)
    orc.update(100)
    worst = max(rel_l2(gpu.get_params(i, w), orc.get_params(i, w)) for i in agents for w in PARAMS6)
    print("config 0, 100 steps in one call: worst network rel-L2 %.3e" % worst)
    assert worst <= 1e-3
    assert gpu.step_count() == 100
    gpu.close()
    gpu, orc, agents = make_pair(0)
    res = free_run_tie_aware(gpu, orc, [(i, i) for i in agents], 100, "config 0")
    print("config 0, 100 steps one at a time: " + describe_free_run(res))
    for i, r in res.items():
        assert r["error"] <= (1e-5 if r["departed"] is None else 1e-3), (i, r)
    gpu.close()


def test_agent_in_population_equals_agent_alone_bit_for_bit():
    hps = workloads.hparams(2, 5)                      # per-agent lr, tau, sigma
    full, _, _ = make_pair(2, P=5, capacity=2000, hps=hps, oracle=False)
    full.update(4)
    for i in (0, 3, 4):
        cfg = pp.make_config(1, 17, 6, (256, 256), 256, 2000)
        alone = pp.Population(cfg, [hps[i]])
        for tr in workloads.transition_chunks(2, i, 2000):
            alone.insert(0, **tr)
        alone.update(4)
        for which in pp.PARAM_CODES:
            if which.startswith("g_") or which.endswith("log_alpha"):
                continue
            assert np.array_equal(full.get_params(i, which), alone.get_params(0, which)), (i, which)
        alone.close()
    full.close()


def test_mixed_policy_delays_and_short_buffers():
    hps = workloads.hparams(2, 3)
    hps[0]["policy_delay"], hps[1]["policy_delay"], hps[2]["policy_delay"] = 1, 2, 3
    gpu, orc, agents = make_pair(2, P=3, capacity=500, fill=100, hps=hps)   # count < batch: with replacement
    gpu.update(7); orc.update(7)
    _compare_state(gpu, orc, agents, 2e-4, "mixed delays, 7 steps", steps=7)
    gpu.close()


def test_ring_buffer_wraps_like_the_oracle():
    cfgd = workloads.CONFIGS[0]
    hps = workloads.hparams(0, 2)
    cfg = pp.make_config(2, 17, 6, (256, 256), 256, 1000)
    gpu = pp.Population(cfg, hps)
    from oracle import td3
    orc = td3.Population(hps, 17, 6, [256, 256], 256, 1000)
    sizes = (300, 900, 1, 2500, 77)                   # wraps, and one insert larger than the ring
    for i in range(2):
        for c, n in enumerate(sizes):
            tr = workloads.transitions(0, i, n, salt=10 + c)
            gpu.insert(i, **tr); orc.insert(i, **tr)
        assert gpu.buffer_count(i) == orc.agents[i].buffer.count == 1000
    gpu.update(1); orc.update(1)
    rows = gpu.debug("batch"); idx = gpu.debug("indices")
    for i in range(2):
        ag = orc.agents[i]
        assert np.array_equal(idx[i].astype(np.int64), ag.last["idx"])
        assert np.array_equal(rows[i], ag.buffer.rows[ag.last["idx"]])
    gpu.close()


def test_device_pointer_insert_for_all_agents_matches_host_insert():
    import torch
    hps = workloads.hparams(0, 2)
    cfg = pp.make_config(2, 17, 6, (256, 256), 256, 700)
    a = pp.Population(cfg, hps); b = pp.Population(cfg, hps)
    n = 900
    trs = [workloads.transitions(0, i, n) for i in range(2)]
    for i in range(2):
        a.insert(i, **trs[i])
    stacked = {k: torch.from_numpy(np.stack([trs[0][k], trs[1][k]])).cuda() for k in trs[0]}
    b.insert(-1, **stacked)
    a.update(2); b.update(2)
    assert np.array_equal(a.debug("batch"), b.debug("batch"))
    for which in ("actor", "critic1", "t_critic2"):
        assert np.array_equal(a.get_params(1, which), b.get_params(1, which))
    a.close(); b.close()


def test_act_matches_oracle_on_ragged_row_counts():
    import torch
    gpu, orc, agents = make_pair(0, capacity=512, fill=512)
    gpu.update(3); orc.update(3)
    rng = np.random.default_rng(5)
    for n in (1, 31, 32, 33, 100):
        obs = rng.standard_normal((2, n, 17)).astype(np.float32)
        ref = orc.act(obs.astype(np.float64))
        got = gpu.act(obs)
        assert got.shape == (2, n, 6)
        assert np.abs(got - ref).max() <= 5e-6
        got_dev = gpu.act(torch.from_numpy(obs).cuda()).cpu().numpy()
        assert np.array_equal(got, got_dev)
    gpu.close()


def test_act_with_exploration_noise_matches_oracle():
    """a = clip(pi(obs) + sigma_i eps, -1, 1): the noise numbers are the same words on both
    sides (element r*A + j of stream 5 at the given counter), so the comparison is
    elementwise: 2e-6 for the Box-Muller float arithmetic times sigma, plus the actor's 5e-6."""
    import torch
    gpu, orc, agents = make_pair(0, capacity=512, fill=512)
    gpu.update(2); orc.update(2)
    rng = np.random.default_rng(6)
    sigma = [0.1, 0.0]                                      # agent 1 acts without noise
    for n, step in ((1, 0), (33, 5), (700, 123456789)):
        obs = rng.standard_normal((2, n, 17)).astype(np.float32)
        ref = orc.act(obs.astype(np.float64), sigma=sigma, step=step)
        got = gpu.act(obs, sigma=sigma, step=step)
        assert np.abs(got - ref).max() <= 1e-5, (n, step, np.abs(got - ref).max())
        assert np.array_equal(got[1], gpu.act(obs)[1])      # sigma 0: exactly the noiseless path
        assert not np.array_equal(got[0], gpu.act(obs)[0])
        got_dev = gpu.act(torch.from_numpy(obs).cuda(), sigma=sigma, step=step).cpu().numpy()
        assert np.array_equal(got, got_dev)                 # device pointers and staged host pieces agree
        assert np.all(np.abs(got) <= 1.0)
    with pytest.raises(pp.PopError):
        gpu.act(obs, sigma=[0.1, -1.0], step=0)
    gpu.close()


def test_errors_from_the_boundary_on_a_live_context():
    gpu, _, _ = make_pair(0, capacity=256, fill=0, oracle=False)
    with pytest.raises(pp.PopError) as e:
        gpu.update(1)
    assert e.value.code == pp.POP_EEMPTY
    with pytest.raises(pp.PopError) as e:
        gpu.get_params(7, "actor")
    assert e.value.code == pp.POP_EINVAL
    small = np.empty(10, dtype=np.float32)
    with pytest.raises(pp.PopError) as e:
        pp.pop_get_params(gpu.ctx, 0, 0, small)
    assert e.value.code == pp.POP_EINVAL
    gpu.close()


def test_every_single_step_from_the_oracle_state_matches_for_100_steps():
    """Step-by-step parity: before each of 100 steps the GPU agents are set to the oracle's
    current state (rounded to fp32), both sides take ONE step, and all parameters, targets
    and Adam moments must agree element by element (gpu_common.check_step_elementwise).  Unlike a
    free-running comparison this is not at the mercy of ReLU patterns that a rounding
    error of 1e-7 flips (after which two correct trajectories drift apart), and it
    exercises every Adam step count, delayed and non-delayed steps and 100 batches."""
    hps = workloads.hparams(1, 10)[:2]                 # per-agent learning rates of the P = 10 config
    gpu, orc, agents = make_pair(1, P=2, capacity=20000, hps=hps)
    gpu.set_debug(1)
    pairs = [(i, i) for i in agents]
    ties, rep = [], None
    for step in range(100):
        force_state(gpu, orc, pairs)
        before = snapshot(orc, agents)
        gpu.update(1)
        orc.update(1)
        rep = check_step_elementwise(gpu, orc, pairs, before, "forced step %d" % step, ties=ties, report=rep)
    print("100 forced steps: %s; %d network updates behind a ReLU tie: %s" % (rep, len(ties), ties))
    assert len(ties) <= 20                               # rare: 600 network updates were compared
    gpu.close()


def test_set_params_round_trips_and_rejects_bad_arguments():
    gpu, _, _ = make_pair(0, capacity=256, fill=256, oracle=False)
    rng = np.random.default_rng(0)
    for which in ("actor", "t_critic2", "v_critic1"):
        n = gpu.actor_size if which.endswith("actor") else gpu.critic_size
        data = rng.standard_normal(n).astype(np.float32)
        gpu.set_params(1, which, data)
        assert np.array_equal(gpu.get_params(1, which), data)
    other = gpu.get_params(0, "actor")
    assert not np.array_equal(other, gpu.get_params(1, "actor"))
    with pytest.raises(pp.PopError) as e:
        gpu.set_params(0, "actor", np.zeros(5, dtype=np.float32))
    assert e.value.code == pp.POP_EINVAL
    with pytest.raises(pp.PopError) as e:
        gpu.set_params(0, "g_actor", np.zeros(gpu.actor_size, dtype=np.float32))
    assert e.value.code == pp.POP_EINVAL
    gpu.close()


def test_launch_structures_agree_bit_for_bit():
    """One launch per step (parts hand results on inside the launch: tagged words for the
    Bellman targets, counters for activation tiles and updated critics), target + critic
    chains fused with and without the rest of the step fused, and one launch per part: identical arithmetic, so every
    parameter and moment must be bit-identical, also for a population size that is not a
    multiple of 8 (uneven XCD groups) and with mixed policy delays (agents whose actor
    parts leave early)."""
    hps = workloads.hparams(2, 11)
    for i, hp in enumerate(hps):
        hp["policy_delay"] = (2, 1, 3)[i % 3]
    states = []
    for launch in (pp.POP_LAUNCH_SINGLE, pp.POP_LAUNCH_TAIL, pp.POP_LAUNCH_TARGET_CRITIC, pp.POP_LAUNCH_PER_PART):
        # rows (16, 64, 16): the class all four structures exist for; full-width tiles in all of them
        gpu, _, _ = make_pair(2, P=11, capacity=3000, hps=hps, oracle=False, launch=launch, rows=(16, 64, 16), half_tiles=1)
        ms, cnt = gpu.update_timed(7)
        assert cnt["gather"] == 1                           # the very first step draws its rows in a launch of its own
        ms, cnt = gpu.update_timed(6)
        assert cnt["gather"] == 0                           # later calls find their rows gathered ahead
        if launch == pp.POP_LAUNCH_SINGLE:
            assert cnt["step"] == 6 and sum(cnt.values()) == 6
        else:
            assert cnt["step"] == 0
            if launch == pp.POP_LAUNCH_TAIL:
                assert cnt["target_critic"] == 6 and cnt["step_tail"] == 6 and sum(cnt.values()) == 12
            elif launch == pp.POP_LAUNCH_TARGET_CRITIC:
                assert cnt["target_critic"] == cnt["wgrad_critic"] == cnt["actor"] == cnt["wgrad_actor"] == 6
                assert sum(cnt.values()) == 24
            else:
                assert cnt["target"] == cnt["critic"] == cnt["wgrad_critic"] == cnt["actor"] == cnt["wgrad_actor"] == 6
                assert sum(cnt.values()) == 30
        assert all(ms[k] > 0.0 for k in ms if cnt[k]) and gpu.step_count() == 13
        gpu.sync()
        states.append({(i, w): gpu.get_params(i, w) for i in range(11) for w in STATE12})
        gpu.close()
    for other in states[1:]:
        for key in states[0]:
            assert np.array_equal(states[0][key], other[key]), key


@pytest.mark.parametrize("P,launches", [(8, {"target_critic": 3, "wgrad_critic": 3}), (9, {"target_critic": 3, "wgrad_critic": 3}),
                                        (12, {"target_critic": 3, "wgrad_critic": 3}), (14, {"target": 3, "critic": 3, "wgrad_critic": 3})])
def test_small_populations_with_32_row_critic_chains_match_oracle(P, launches):
    """Up to 8 agents the critic chains take 32 rows beside the 16-row target chains of the same launch; with 9
    and 10 the target workgroups run critic 1 for their own rows and only critic 2 has 32-row workgroups (64-row
    ones with 11 and 12 agents); from 13 to 16 agents the two chains are launches of their own.  Both against the oracle over three steps with mixed
    policy delays, in the launch structure the library picks by itself; a single launch per step is refused for
    these row classes."""
    hps = workloads.hparams(2, P)
    for i, hp in enumerate(hps):
        hp["policy_delay"] = (2, 1, 3)[i % 3]
    gpu, orc, _ = make_pair(2, P=P, capacity=1500, hps=hps)
    _, cnt = gpu.update_timed(3)
    for k, v in launches.items():
        assert cnt[k] == v, (k, cnt)
    assert cnt["step"] == 0
    orc.update(3)
    _compare_state(gpu, orc, range(P), 1e-4, "P = %d, 3 steps" % P, steps=3)
    gpu.close()
    if P == 9:                                          # falls back to 64-row critic chains, which the single launch has
        make_pair(2, P=P, capacity=1500, hps=hps, oracle=False, launch=pp.POP_LAUNCH_SINGLE)[0].close()
        return
    with pytest.raises(pp.PopError) as e:
        make_pair(2, P=P, capacity=1500, hps=hps, oracle=False, launch=pp.POP_LAUNCH_SINGLE)
    assert e.value.code == pp.POP_EINVAL


def test_sixty_four_row_chains_match_oracle_and_each_other():
    """No population gets 64-row target and actor chains by default any more (the 32-row ones overtook them);
    tuning.rows_* = 64 still selects them.  P = 5 with mixed delays, 5 steps: against the oracle, and one launch per step
    against one launch per part bit for bit (full-width tiles in all of them)."""
    hps = workloads.hparams(2, 5)
    for i, hp in enumerate(hps):
        hp["policy_delay"] = (2, 1, 3)[i % 3]
    states = []
    for launch in (pp.POP_LAUNCH_TARGET_CRITIC, pp.POP_LAUNCH_SINGLE, pp.POP_LAUNCH_PER_PART):
        gpu, orc, _ = make_pair(2, P=5, capacity=2000, hps=hps, oracle=(launch == pp.POP_LAUNCH_TARGET_CRITIC),
                                launch=launch, rows=64, half_tiles=1)
        gpu.update(5)
        if orc is not None:
            orc.update(5)
            _compare_state(gpu, orc, range(5), 1e-4, "64-row chains, 5 steps", steps=5)
        gpu.sync()
        states.append({(i, w): gpu.get_params(i, w) for i in range(5) for w in STATE12})
        gpu.close()
    for other in states[1:]:
        for key in states[0]:
            assert np.array_equal(states[0][key], other[key]), key


def test_mid_size_single_launch_with_mixed_delays_equals_separate_launches():
    """The single launch of mid-size populations (32-row chains, two workgroups per CU): only critic 1 of an agent whose
    actor part runs on this step stores its parameters through to memory and counts in for the actor chain that waits
    for it; with delays 2, 1 and 3 side by side every step has agents of both kinds.  Bit for bit against the
    structures that hand over at launch boundaries, P = 40 (the single launch is the default there), 7 steps."""
    hps = workloads.hparams(2, 40)
    for i, hp in enumerate(hps):
        hp["policy_delay"] = (2, 1, 3)[i % 3]
    states = []
    for launch in (pp.POP_LAUNCH_SINGLE, pp.POP_LAUNCH_TAIL, pp.POP_LAUNCH_TARGET_CRITIC):
        gpu, _, _ = make_pair(2, P=40, capacity=1000, hps=hps, oracle=False, launch=launch)
        assert gpu.tuning()["launch"] == launch and gpu.tuning()["rows_actor"] == 32
        gpu.update(7)
        gpu.sync()
        states.append({(i, w): gpu.get_params(i, w) for i in range(40) for w in STATE12})
        gpu.close()
    for other in states[1:]:
        for key in states[0]:
            assert np.array_equal(states[0][key], other[key]), key


def test_tile_width_is_independent_of_the_launch_structure():
    """Half-width weight-gradient tiles (the default up to 10 agents) sum the batch in two halves: results differ from
    full-width tiles in the last bits only, whichever launch structure runs them, and do not depend on anything but
    the tuning field."""
    hps = workloads.hparams(2, 4)
    out = {}
    for half in (0, 1, 2):
        for launch in (pp.POP_LAUNCH_AUTO, pp.POP_LAUNCH_PER_PART):
            gpu, _, _ = make_pair(2, P=4, capacity=1200, hps=hps, oracle=False, launch=launch, rows=(16, 32, 16), half_tiles=half, actor_ahead=1)
            gpu.update(3)
            out[half, launch] = {(i, w): gpu.get_params(i, w) for i in range(4) for w in STATE12}
            gpu.close()
    for half in (0, 1, 2):                                  # same tile width: launch structures agree bit for bit
        a, b = out[half, pp.POP_LAUNCH_AUTO], out[half, pp.POP_LAUNCH_PER_PART]
        assert all(np.array_equal(a[k], b[k]) for k in a)
    a, b, c = out[0, pp.POP_LAUNCH_AUTO], out[2, pp.POP_LAUNCH_AUTO], out[1, pp.POP_LAUNCH_AUTO]
    assert all(np.array_equal(a[k], b[k]) for k in a)       # "choose" means on at P = 4
    assert any(not np.array_equal(a[k], c[k]) for k in a)   # and full-width tiles differ ...
    assert max(rel_l2(a[k], c[k]) for k in a if c[k].any()) <= 1e-5   # ... in rounding only


@pytest.mark.parametrize("P", [4, 10])
def test_actor_forward_inside_the_target_critic_launch_changes_rounding_only(P):
    """Small populations run the actor's own forward pass in the critic-2 workgroups of the target / critic launch
    (tuning.actor_ahead; the default at 9 and 10 agents), on 32-row instead of 16-row tiles: against the same steps with the
    forward pass in the actor launch the results differ, and in the order of the fp32 sums only.  Agents with
    different policy delays take it on their own delayed steps."""
    hps = workloads.hparams(2, P)
    for i, h in enumerate(hps):
        h["policy_delay"] = 1 + i % 3
    out = {}
    for ahead in (0, 1, 2):
        gpu, _, _ = make_pair(2, P=P, capacity=1200, hps=hps, oracle=False, actor_ahead=ahead)
        gpu.update(4)
        out[ahead] = {(i, w): gpu.get_params(i, w) for i in range(P) for w in STATE12}
        gpu.close()
    chosen = 2 if P == 10 else 1                              # "choose": on where the target workgroups run critic 1
    assert all(np.array_equal(out[0][k], out[chosen][k]) for k in out[0])
    assert any(not np.array_equal(out[1][k], out[2][k]) for k in out[1])
    worst = max(rel_l2(out[2][k], out[1][k]) for k in out[1] if out[1][k].any())
    assert worst <= 2e-5, worst


def test_copy_agent_and_set_hparams_follow_the_oracle():
    """The population step of App. B.1 on both sides: train, replace agent 0 by a copy of
    agent 2 (with its buffer) and agent 1 by a copy of agent 3 (keeping its own buffer), give
    the copies new hyperparameters (learning rates, discount, noise, a different policy
    delay), train on.  Parameters, targets and moments are compared after the copy (bit for
    bit against the parent on the GPU), one step later (1e-4) and a few steps later."""
    P = 4
    hps = workloads.hparams(2, P)
    gpu, orc, _ = make_pair(2, P=P, capacity=3000, hps=hps)
    for side in (gpu, orc):
        side.update(5)
        side.copy_agent(0, 2, True)
        side.copy_agent(1, 3, False)
    for w in STATE12:
        assert np.array_equal(gpu.get_params(0, w), gpu.get_params(2, w)), w
        assert np.array_equal(gpu.get_params(1, w), gpu.get_params(3, w)), w
    assert gpu.buffer_count(0) == gpu.buffer_count(2) == 3000
    new0 = dict(hps[0], lr_actor=1e-3, lr_critic=2e-4, gamma=0.95, policy_noise=0.4, noise_clip=0.3, policy_delay=3)
    new1 = dict(hps[1], lr_actor=5e-5, lr_critic=1e-3, tau=0.01, policy_delay=1, seed=987654321)
    for side in (gpu, orc):
        side.set_hparams(0, new0)
        side.set_hparams(1, new1)
    pairs = [(i, i) for i in range(P)]
    gpu.set_debug(1)
    ties = []
    force_state(gpu, orc, pairs)                               # remove the drift of the first 5 steps
    before = snapshot(orc, range(P))
    gpu.update(1); orc.update(1)                               # t = 5: actor step only for agent 1 (delay 1)
    check_step_elementwise(gpu, orc, pairs, before, "first step after copy + new hyperparameters", ties=ties)
    force_state(gpu, orc, pairs)
    before = snapshot(orc, range(P))
    gpu.update(1); orc.update(1)                               # t = 6: actor step for agents 0 (delay 3), 1, 2, 3
    check_step_elementwise(gpu, orc, pairs, before, "second step (actor step under the new delay; Adam count continues)", ties=ties)
    gpu.set_debug(0)
    assert orc.agents[0].actor_updates == 4 and orc.agents[1].actor_updates == 5
    gpu.update(6); orc.update(6)
    _compare_state(gpu, orc, range(P), 1e-3, "six more free steps", steps=6)
    with pytest.raises(pp.PopError):
        gpu.copy_agent(0, P, True)
    with pytest.raises(pp.PopError):
        gpu.set_hparams(0, dict(new0, policy_delay=0))
    with pytest.raises(pp.PopError):
        gpu.set_hparams(0, dict(new0, seed=0))
    gpu.close()


# ---------------------------------------------------------------------------------------------
# Wider shapes (plain TD3): Ant-v2 (obs 111, act 8: critic fan-in 119), the widest fan-in the chains take (obs 440,
# act 8), Humanoid-v2 (obs 376, act 17: scratch rows of 24 floats, a head the split contraction does not cover) and one
# in between (obs 40, act 10: wide scratch rows on a narrow input).  The first layers run software-pipelined (the
# chains of the SAC Humanoid shapes), every part of the step is a launch of its own.
WIDE = [(111, 8), (440, 8), (376, 17), (40, 10)]


@pytest.mark.parametrize("obs_dim,act_dim", WIDE)
def test_wide_observations_forced_single_steps_match_oracle(obs_dim, act_dim):
    hps = workloads.hparams(1, 10)[:2]
    gpu, orc, agents = make_pair(1, P=2, capacity=700, hps=hps, obs_dim=obs_dim, act_dim=act_dim)
    for i in agents:
        for w in PARAMS6:
            assert np.array_equal(gpu.get_params(i, w), orc.get_params(i, w).astype(np.float32)), (i, w)
    gpu.set_debug(1)
    pairs = [(i, i) for i in agents]
    ties, rep = [], None
    for step in range(12):
        force_state(gpu, orc, pairs)
        before = snapshot(orc, agents)
        gpu.update(1); orc.update(1)
        rep = check_step_elementwise(gpu, orc, pairs, before, "forced step %d at obs %d, act %d" % (step, obs_dim, act_dim),
                                     ties=ties, report=rep)
        idx = gpu.debug("indices")
        for i in agents:
            assert np.array_equal(idx[i].astype(np.int64), orc.agents[i].last["idx"])
    print("12 forced steps at obs %d, act %d: %s; %d network updates behind a ReLU tie: %s" % (obs_dim, act_dim, rep, len(ties), ties))
    assert len(ties) <= 8
    gpu.close()


@pytest.mark.parametrize("obs_dim,act_dim", WIDE)
def test_wide_observations_in_a_mid_size_population(obs_dim, act_dim):
    """P = 20 (32-row chains): agents 0 and 19 against the oracle, the first step element by element, three more free
    steps per tensor (Adam's first steps are sign-like: entries of the wide first layers whose gradient is within
    rounding of zero may start the other way, which the element-wise check accounts for entry by entry and the free
    run can only bound), and acting."""
    hps = workloads.hparams(2, 20)
    gpu, orc, agents = make_pair(2, P=20, capacity=400, hps=hps, agents=[0, 19], obs_dim=obs_dim, act_dim=act_dim)
    gpu.set_debug(1)
    pairs = list(zip(agents, range(len(agents))))
    before = snapshot(orc, range(len(agents)))
    gpu.update(1); orc.update(1)
    ties = []
    rep = check_step_elementwise(gpu, orc, pairs, before, "first step at P = 20, obs %d, act %d" % (obs_dim, act_dim), ties=ties)
    print("first step at P = 20, obs %d, act %d: %s; ties %s" % (obs_dim, act_dim, rep, ties))
    gpu.update(3); orc.update(3)
    check_tensors_all(gpu, orc, pairs, PARAMS6, 1e-3, "four steps at P = 20, obs %d, act %d" % (obs_dim, act_dim), steps=4)
    force_state(gpu, orc, pairs)                            # acting: the same actors on both sides
    rng = np.random.default_rng(9)
    obs = rng.standard_normal((20, 45, obs_dim)).astype(np.float32)
    got = gpu.act(obs)
    for i, j in pairs:
        want = orc.agents[j].act(obs[i].astype(np.float64))
        assert float(np.abs(got[i] - want).max()) <= 2e-5
    gpu.close()

