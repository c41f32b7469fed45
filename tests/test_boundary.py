"""CPU-only checks of the C boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2206_08888_amd as pp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pp.lib_path()):
        from paper_2206_08888_amd import build
        build.build()
    return pp.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "pop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pop_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_the_header(lib):
    assert C.sizeof(pp.pop_hparams) == 64
    assert C.sizeof(pp.pop_config) == 48


def test_workspace_size_and_net_sizes(lib):
    cfg = pp.make_config(2, 17, 6, (256, 256), 256, 10000)
    assert pp.pop_net_size(cfg, pp.PARAM_CODES["actor"]) == 17 * 256 + 256 + 256 * 256 + 256 + 256 * 6 + 6 == 71942
    assert pp.pop_net_size(cfg, pp.PARAM_CODES["critic2"]) == 72193
    small = pp.pop_workspace_bytes(cfg)
    big = pp.pop_workspace_bytes(pp.make_config(2, 17, 6, (256, 256), 256, 20000))
    assert big - small == 2 * 10000 * 42 * 4            # replay rows are 2*17 + 6 + 2 floats
    assert small % 256 == 0


@pytest.mark.parametrize("kwargs,code", [
    (dict(P=0), pp.POP_EINVAL),
    (dict(batch=0), pp.POP_EINVAL),
    (dict(capacity=0), pp.POP_EINVAL),
    (dict(hidden=(128, 128)), pp.POP_EUNSUPPORTED),
    (dict(hidden=(256,)), pp.POP_EUNSUPPORTED),
    (dict(batch=100), pp.POP_EUNSUPPORTED),
    (dict(obs_dim=100), pp.POP_EUNSUPPORTED),
    (dict(act_dim=9), pp.POP_EUNSUPPORTED),
    (dict(capacity=1 << 33), pp.POP_EUNSUPPORTED),
    (dict(algo=7), pp.POP_EINVAL),
    (dict(algo=pp.POP_ALGO_SAC, obs_dim=100, act_dim=25), pp.POP_EUNSUPPORTED),
    (dict(algo=pp.POP_ALGO_SAC, obs_dim=440, act_dim=17), pp.POP_EUNSUPPORTED),
])
def test_bad_configs_are_rejected(lib, kwargs, code):
    base = dict(P=2, obs_dim=17, act_dim=6, hidden=(256, 256), batch=256, capacity=1000)
    base.update(kwargs)
    with pytest.raises(pp.PopError) as e:
        pp.pop_workspace_bytes(pp.make_config(**base))
    assert e.value.code == code
    assert pp.pop_last_error() != ""


def test_sac_takes_the_humanoid_shapes(lib):
    cfg = pp.make_config(2, 376, 17, (256, 256), 256, 1000, algo=pp.POP_ALGO_SAC)
    assert pp.pop_net_size(cfg, pp.PARAM_CODES["actor"]) == 376 * 256 + 256 + 256 * 256 + 256 + 256 * 34 + 34
    assert pp.pop_net_size(cfg, pp.PARAM_CODES["critic1"]) == 393 * 256 + 256 + 256 * 256 + 256 + 256 + 1
    assert pp.pop_workspace_bytes(cfg) > 2 * 1000 * (2 * 376 + 17 + 2) * 4


def test_create_checks_arguments_before_any_gpu_work(lib):
    import workloads
    cfg = pp.make_config(2, 17, 6, (256, 256), 256, 1000)
    hp = pp.make_hparams(workloads.hparams(0, 2))
    need = pp.pop_workspace_bytes(cfg)
    with pytest.raises(pp.PopError) as e:               # NULL workspace
        pp.pop_create(cfg, hp, 0, 0, need, 0)
    assert e.value.code == pp.POP_EINVAL
    with pytest.raises(pp.PopError) as e:               # misaligned workspace
        pp.pop_create(cfg, hp, 0, 0x1000 + 8, need, 0)
    assert e.value.code == pp.POP_EINVAL
    with pytest.raises(pp.PopError) as e:               # too small
        pp.pop_create(cfg, hp, 0, 0x10000, need - 1, 0)
    assert e.value.code == pp.POP_ENOMEM
    bad = workloads.hparams(0, 2)
    bad[1]["policy_delay"] = 0
    with pytest.raises(pp.PopError) as e:
        pp.pop_create(cfg, pp.make_hparams(bad), 0, 0x10000, need, 0)
    assert e.value.code == pp.POP_EINVAL and "policy_delay" in str(e.value)


def test_null_context_is_an_error_not_a_crash(lib):
    assert lib.pop_update(None, 1) == pp.POP_EINVAL
    assert lib.pop_sync(None) == pp.POP_EINVAL
    assert lib.pop_destroy(None) == pp.POP_EINVAL
    assert lib.pop_step_count(None) == pp.POP_EINVAL
