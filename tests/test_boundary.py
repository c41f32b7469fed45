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


def test_struct_sizes_match_the_header(lib, tmp_path):
    """The ctypes structures against the header itself: a C program compiled from include/pop.h prints its sizes
    and the offsets of the fields that follow padding."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "pop.h"\n'
                   'int main(void) { printf("%zu %zu %zu %zu %zu\\n", sizeof(pop_hparams), sizeof(pop_config), sizeof(pop_tuning), '
                   'offsetof(pop_config, capacity), offsetof(pop_config, tuning)); return 0; }\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got == [C.sizeof(pp.pop_hparams), C.sizeof(pp.pop_config), C.sizeof(pp.pop_tuning),
                   pp.pop_config.capacity.offset, pp.pop_config.tuning.offset] == [64, 80, 28, 40, 48]


def test_bad_tuning_values_are_refused_before_any_gpu_work(lib):
    for kw in (dict(launch=7), dict(launch=-1), dict(rows=(16, 16, 16)), dict(rows=48), dict(half_tiles=3), dict(rows_critic1=32), dict(actor_ahead=3)):
        with pytest.raises(pp.PopError) as e:
            pp.pop_workspace_bytes(pp.make_config(2, 17, 6, (256, 256), 256, 100, **kw))
        assert e.value.code == pp.POP_EINVAL and "tuning" in str(e.value), kw
    # the rows per workgroup size the partial-sum areas of the workspace
    a = pp.pop_workspace_bytes(pp.make_config(20, 17, 6, (256, 256), 256, 100, rows=64))
    b = pp.pop_workspace_bytes(pp.make_config(20, 17, 6, (256, 256), 256, 100, rows=32))
    assert a < b


def test_nothing_is_read_from_the_environment(lib, monkeypatch):
    """The launch structure and tile geometry come from pop_config.tuning alone."""
    cfg = pp.make_config(20, 17, 6, (256, 256), 256, 100)
    plain = pp.pop_workspace_bytes(cfg)
    for name, value in (("POP_ROWS", "64"), ("POP_FUSE", "0"), ("POP_HALF_TILES", "1")):
        monkeypatch.setenv(name, value)
    assert pp.pop_workspace_bytes(cfg) == plain
    text = "".join(open(os.path.join(ROOT, "paper_2206_08888_amd", "csrc", f)).read()
                   for f in os.listdir(os.path.join(ROOT, "paper_2206_08888_amd", "csrc")))
    assert "getenv" not in text


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
    (dict(obs_dim=443), pp.POP_EUNSUPPORTED),
    (dict(act_dim=25), pp.POP_EUNSUPPORTED),
    (dict(algo=pp.POP_ALGO_TD3_SHARED, obs_dim=443), pp.POP_EUNSUPPORTED),
    (dict(algo=pp.POP_ALGO_TD3_SHARED, act_dim=25), pp.POP_EUNSUPPORTED),
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


def test_td3_takes_the_humanoid_shapes(lib):
    cfg = pp.make_config(2, 376, 17, (256, 256), 256, 1000)
    assert pp.pop_net_size(cfg, pp.PARAM_CODES["actor"]) == 376 * 256 + 256 + 256 * 256 + 256 + 256 * 17 + 17
    assert pp.pop_net_size(cfg, pp.PARAM_CODES["critic2"]) == 393 * 256 + 256 + 256 * 256 + 256 + 256 + 1


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
