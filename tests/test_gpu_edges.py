"""GPU parity at the edges of the supported shapes: the largest and the smallest observation / action sizes of
each algorithm, buffers shorter than a batch, zero-step calls.  Tolerances as elsewhere: the first step and three
forced single steps element by element (gpu_common.check_step_elementwise; at large fan-ins a hidden unit within
fp32 rounding of its kink is common, and must then be demonstrated as such)."""
import numpy as np
import pytest

import paper_2206_08888_amd as pp
import workloads
from gpu_common import STATE12, PARAMS6, check_step_elementwise, check_tensors_all, ensure_built, rel_l2, snapshot
from oracle import sac as oracle_sac, td3 as oracle_td3, td3_shared as oracle_shared

pytestmark = pytest.mark.gpu

SAC_NETS = ("actor", "critic1", "critic2", "t_critic1", "t_critic2")
SAC_STATE = SAC_NETS + ("m_actor", "m_critic1", "m_critic2", "v_actor", "v_critic1", "v_critic2",
                        "log_alpha", "m_log_alpha", "v_log_alpha")


@pytest.fixture(scope="module", autouse=True)
def _lib():
    ensure_built()


def _pair(algo, P, O, A, capacity, fill=None, hps=None, **tuning):
    fill = capacity if fill is None else fill
    hps = workloads.hparams(2, P) if hps is None else hps
    if algo == "sac":
        for hp in hps:
            hp["target_entropy"] = -float(A)
    code = {"td3": pp.POP_ALGO_TD3, "sac": pp.POP_ALGO_SAC, "shared": pp.POP_ALGO_TD3_SHARED}[algo]
    gpu = pp.Population(pp.make_config(P, O, A, (256, 256), 256, capacity, algo=code, **tuning), hps)
    mod = {"td3": oracle_td3, "sac": oracle_sac, "shared": oracle_shared}[algo]
    orc = mod.Population(hps, O, A, [256, 256], 256, capacity)
    for i in range(P):
        tr = workloads.transitions(2, i, fill, obs_dim=O, act_dim=A, salt=3)
        gpu.insert(i, **tr)
        orc.insert(i, **tr)
    return gpu, orc


def _worst(gpu, orc, P, names):
    return max(rel_l2(gpu.get_params(i, n), orc.get_params(i, n)) for i in range(P) for n in names)


def _first_then_forced(gpu, orc, P, state, label, steps=3):
    """The first step from the initial state and `steps` forced single steps, each element by element."""
    gpu.set_debug(1)
    pairs = [(i, i) for i in range(P)]
    ties, rep = [], None
    for k in range(1 + steps):
        if k:
            for i in range(P):
                for n in state:
                    gpu.set_params(i, n, orc.get_params(i, n))
        before = snapshot(orc, range(P))
        gpu.update(1); orc.update(1)
        rep = check_step_elementwise(gpu, orc, pairs, before, "%s, step %d" % (label, k), ties=ties, report=rep)
    gpu.set_debug(0)
    return rep, ties


@pytest.mark.parametrize("O,A", [(56, 8), (1, 1), (63, 1)])
def test_td3_at_the_ends_of_its_shape_range(O, A):
    gpu, orc = _pair("td3", 3, O, A, 600)
    for i in range(3):
        for n in PARAMS6:
            assert np.array_equal(gpu.get_params(i, n), orc.get_params(i, n).astype(np.float32)), (i, n)
    rep, ties = _first_then_forced(gpu, orc, 3, STATE12, "TD3 obs %d act %d" % (O, A))
    obs = np.random.default_rng(2).standard_normal((3, 37, O)).astype(np.float32)
    assert np.abs(gpu.act(obs) - orc.act(obs.astype(np.float64))).max() <= 1e-5
    print("TD3 obs %d act %d: %s; ties %s" % (O, A, rep, ties))
    gpu.close()


@pytest.mark.parametrize("O,A,P", [(424, 24, 2), (424, 24, 20), (1, 1, 2), (60, 4, 2), (61, 4, 2)])
def test_sac_at_the_ends_of_its_shape_range(O, A, P):
    """(424, 24) is the largest input and head the SAC kernels take (16-row chains at P = 2, 32-row ones at P = 20);
    (60, 4) / (61, 4) sit on either side of the switch to the pipelined first layers."""
    gpu, orc = _pair("sac", P, O, A, 400)
    for i in range(P):
        for n in SAC_NETS:
            assert np.array_equal(gpu.get_params(i, n), orc.get_params(i, n).astype(np.float32)), (i, n)
    rep, ties = _first_then_forced(gpu, orc, P, SAC_STATE, "SAC obs %d act %d P %d" % (O, A, P))
    for i in range(P):
        assert abs(float(gpu.get_params(i, "log_alpha")[0]) - float(orc.get_params(i, "log_alpha")[0])) <= 2e-6
    obs = np.random.default_rng(2).standard_normal((P, 19, O)).astype(np.float32)
    assert np.abs(gpu.act(obs) - orc.act(obs.astype(np.float64))).max() <= (2e-5 if O > 64 else 5e-6)
    print("SAC obs %d act %d P %d: %s; ties %s" % (O, A, P, rep, ties))
    gpu.close()


@pytest.mark.parametrize("algo", ["td3", "sac", "shared"])
def test_buffers_shorter_than_a_batch_and_zero_step_calls(algo):
    """100 transitions for a batch of 256: sampling is with replacement over the filled part; update(0) is a no-op."""
    P = 3
    gpu, orc = _pair(algo, P, 17, 6, 500, fill=100)
    nets = SAC_NETS if algo == "sac" else PARAMS6
    before = {(i, n): gpu.get_params(i, n) for i in range(P) for n in nets}
    gpu.update(0)
    assert gpu.step_count() == 0
    for (i, n), v in before.items():
        assert np.array_equal(gpu.get_params(i, n), v)
    gpu.update(2); orc.update(2)
    idx = gpu.debug("indices")
    for i in range(P):
        assert idx[i].max() < 100
        assert np.array_equal(idx[i].astype(np.int64), orc.agents[i].last["idx"]), i
    assert _worst(gpu, orc, P, nets) <= 1e-4
    if algo == "shared":
        check_tensors_all(gpu, orc, [(0, 0)], PARAMS6, 1e-4, "short buffers", steps=2)
        check_tensors_all(gpu, orc, [(i, i) for i in range(P)], ("actor", "t_actor"), 1e-4, "short buffers", steps=2)
    else:
        check_tensors_all(gpu, orc, [(i, i) for i in range(P)], nets, 1e-4, "short buffers", steps=2)
    gpu.close()


def test_unsupported_shapes_are_refused_with_a_message():
    for algo, O, A in ((pp.POP_ALGO_TD3, 441, 8), (pp.POP_ALGO_TD3, 17, 25), (pp.POP_ALGO_TD3_SHARED, 440, 9), (pp.POP_ALGO_TD3_SHARED, 17, 25),
                       (pp.POP_ALGO_SAC, 425, 24), (pp.POP_ALGO_SAC, 100, 25)):
        with pytest.raises(pp.PopError) as e:
            pp.Population(pp.make_config(2, O, A, (256, 256), 256, 100, algo=algo), workloads.hparams(2, 2))
        assert e.value.code == pp.POP_EUNSUPPORTED and "must be <=" in str(e.value)


def test_row_classes_without_a_kernel_are_refused_at_launch():
    """tuning.rows_* can ask for (target, critic, actor) rows per workgroup that the fused launches have no kernel for:
    the launch is refused with an error, nothing runs; as separate launches the same rows work and match."""
    gpu, orc = _pair("td3", 3, 17, 6, 600, rows=(32, 64, 32), launch=pp.POP_LAUNCH_SINGLE)
    with pytest.raises(pp.PopError) as e:
        gpu.update(1)
    assert e.value.code == pp.POP_EHIP
    gpu.close()
    gpu, orc = _pair("td3", 3, 17, 6, 600, rows=(32, 64, 32), launch=pp.POP_LAUNCH_PER_PART)
    gpu.update(2); orc.update(2)
    assert _worst(gpu, orc, 3, PARAMS6) <= 1e-4
    check_tensors_all(gpu, orc, [(i, i) for i in range(3)], PARAMS6, 1e-4, "separate launches", steps=2)
    gpu.close()


def test_critic1_inside_the_target_workgroups_needs_the_fused_launch():
    with pytest.raises(pp.PopError) as e:                   # TD3, target and critic chains in one launch only
        _pair("td3", 3, 17, 6, 300, rows=(16, 32, 16), rows_critic1=16, launch=pp.POP_LAUNCH_PER_PART)
    assert e.value.code == pp.POP_EINVAL
    with pytest.raises(pp.PopError) as e:                   # the actor's forward pass ahead: in that launch only
        _pair("td3", 3, 17, 6, 300, launch=pp.POP_LAUNCH_PER_PART, actor_ahead=2)
    assert e.value.code == pp.POP_EINVAL


def test_the_tuning_in_force_is_reported():
    """pop_get_tuning resolves every "choose": the population classes of the library's own choice, and a caller's
    fields handed back as given."""
    def tuning(algo, P, **kw):
        gpu = pp.Population(pp.make_config(P, 17, 6, (256, 256), 256, 64, algo=algo, **kw), workloads.hparams(2, P))
        t = gpu.tuning()
        gpu.close()
        return t
    t = tuning(pp.POP_ALGO_TD3, 10)
    assert t == dict(launch=pp.POP_LAUNCH_TARGET_CRITIC, rows_target=16, rows_critic=32, rows_actor=16, rows_critic1=16,
                     half_tiles=2, actor_ahead=2)
    t = tuning(pp.POP_ALGO_TD3, 4)
    assert (t["launch"], t["rows_critic1"], t["actor_ahead"], t["half_tiles"]) == (pp.POP_LAUNCH_TARGET_CRITIC, 32, 1, 2)
    t = tuning(pp.POP_ALGO_TD3, 80)
    assert t == dict(launch=pp.POP_LAUNCH_SINGLE, rows_target=32, rows_critic=32, rows_actor=32, rows_critic1=32,
                     half_tiles=1, actor_ahead=1)
    t = tuning(pp.POP_ALGO_TD3, 6, launch=pp.POP_LAUNCH_PER_PART, rows=(32, 64, 32), half_tiles=1)
    assert t == dict(launch=pp.POP_LAUNCH_PER_PART, rows_target=32, rows_critic=64, rows_actor=32, rows_critic1=64,
                     half_tiles=1, actor_ahead=1)
    assert tuning(pp.POP_ALGO_SAC, 32)["launch"] == pp.POP_LAUNCH_PER_PART


@pytest.mark.parametrize("launch,rows", [(pp.POP_LAUNCH_TARGET_CRITIC, None), (pp.POP_LAUNCH_SINGLE, (16, 64, 16))])
def test_a_wait_between_workgroups_that_runs_out_is_reported_once_and_the_context_recovers(launch, rows):
    """Workgroups of a fused launch wait for results of other workgroups of the same launch, each wait bounded by
    the constant-rate clock.  With the bound set to one tick (10 ns) from the host every such wait gives up at
    once: the kernels still run to their end (with stale operands), the step's results are invalid, and the next
    call that synchronises says so -- once.  After the state is restored the context works as before."""
    hps = workloads.hparams(2, 4)
    def make():
        gpu = pp.Population(pp.make_config(4, 17, 6, (256, 256), 256, 800, launch=launch, rows=rows, half_tiles=1), hps)
        for i in range(4):
            gpu.insert(i, **workloads.transitions(2, i, 800))
        return gpu
    gpu, twin = make(), make()
    gpu.update(2); twin.update(2)
    saved = {(i, w): gpu.get_params(i, w) for i in range(4) for w in STATE12}
    gpu.set_option(pp.POP_OPT_WAIT_LIMIT_TICKS, 1)
    gpu.update(1)
    with pytest.raises(pp.PopError) as e:
        gpu.sync()
    assert e.value.code == pp.POP_EHIP and "time limit" in str(e.value)
    gpu.sync()                                              # reported once, then cleared
    gpu.update(1)                                           # still one tick: the other reporting path
    with pytest.raises(pp.PopError) as e:
        gpu.get_params(0, "actor")
    assert e.value.code == pp.POP_EHIP
    gpu.get_params(0, "actor")
    with pytest.raises(pp.PopError):
        gpu.set_option(pp.POP_OPT_WAIT_LIMIT_TICKS, 0)
    with pytest.raises(pp.PopError):
        gpu.set_option(99, 1)
    gpu.set_option(pp.POP_OPT_WAIT_LIMIT_TICKS, 5_000_000)
    gpu.close()
    # a fresh context (the step counter of the faulted one has moved on) with the saved state continues like the twin
    again = make()
    again.update(2)
    for (i, w), v in saved.items():
        assert np.array_equal(again.get_params(i, w), v)
    again.update(3); twin.update(3)
    for i in range(4):
        for w in STATE12:
            assert np.array_equal(again.get_params(i, w), twin.get_params(i, w)), (i, w)
    again.close(); twin.close()
