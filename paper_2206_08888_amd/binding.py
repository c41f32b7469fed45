"""ctypes binding of include/pop.h: same names, argument marshalling only.

Nothing here computes: every step of the update runs in the HIP kernels of
libpop.so.  If the library has not been built the import of the library fails
loudly; there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

POP_OK, POP_EINVAL, POP_ENOMEM, POP_EEMPTY, POP_EHIP, POP_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
POP_ALGO_TD3, POP_ALGO_SAC, POP_ALGO_TD3_SHARED = 0, 1, 2

PARAM_CODES = {
    "actor": 0, "critic1": 1, "critic2": 2, "t_actor": 3, "t_critic1": 4, "t_critic2": 5,
    "m_actor": 6, "m_critic1": 7, "m_critic2": 8, "v_actor": 9, "v_critic1": 10, "v_critic2": 11,
    "g_actor": 12, "g_critic1": 13, "g_critic2": 14,
    "log_alpha": 15, "m_log_alpha": 16, "v_log_alpha": 17,        # SAC only, one float each
}
DEBUG_CODES = {"indices": 0, "batch": 1, "target_action": 2, "target_y": 3, "losses": 4}


class pop_hparams(C.Structure):
    _fields_ = [("seed", C.c_uint64),
                ("lr_actor", C.c_float), ("lr_critic", C.c_float), ("gamma", C.c_float), ("tau", C.c_float),
                ("policy_noise", C.c_float), ("noise_clip", C.c_float), ("policy_delay", C.c_int32),
                ("adam_b1", C.c_float), ("adam_b2", C.c_float), ("adam_eps", C.c_float),
                ("lr_alpha", C.c_float), ("target_entropy", C.c_float), ("init_log_alpha", C.c_float),
                ("reserved_", C.c_int32)]


POP_LAUNCH_AUTO, POP_LAUNCH_PER_PART, POP_LAUNCH_TARGET_CRITIC, POP_LAUNCH_SINGLE, POP_LAUNCH_TAIL = 0, 1, 2, 3, 4
POP_OPT_WAIT_LIMIT_TICKS = 0


class pop_tuning(C.Structure):
    _fields_ = [("launch", C.c_int32), ("rows_target", C.c_int32), ("rows_critic", C.c_int32), ("rows_actor", C.c_int32),
                ("rows_critic1", C.c_int32), ("half_tiles", C.c_int32), ("actor_ahead", C.c_int32)]


class pop_config(C.Structure):
    _fields_ = [("algo", C.c_int32), ("P", C.c_int32), ("obs_dim", C.c_int32), ("act_dim", C.c_int32),
                ("n_hidden", C.c_int32), ("hidden", C.c_int32 * 4), ("batch", C.c_int32),
                ("capacity", C.c_int64), ("tuning", pop_tuning)]


assert C.sizeof(pop_hparams) == 64 and C.sizeof(pop_config) == 80


class PopError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("pop error %d: %s" % (code, message))
        self.code = code


_LIB = None


def lib_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpop.so")


def load_library(path=None):
    """Load libpop.so (built by `python -m paper_2206_08888_amd.build`), or, when the first call of the process names
    it, another build of the same boundary (the traced libpop_trace.so)."""
    global _LIB
    if _LIB is not None:
        assert path is None or os.path.samefile(path, _LIB._name), "another build of the library is already loaded"
        return _LIB
    # PyTorch ships its own HIP runtime; callers allocate the workspace and the stream with it, so it has to be the
    # runtime libpop.so binds to as well: loaded first, its libamdhip64 satisfies the library's dependency.  (Loaded
    # the other way round the process holds two runtimes and the library's one finds no device.)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    path = lib_path() if path is None else path
    if not os.path.exists(path):
        raise ImportError("%s is missing: build it with `python -m paper_2206_08888_amd.build` "
                          "(there is no fallback implementation)" % path)
    lib = C.CDLL(path)
    vp, fp, i32, i64, u64 = C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    cfgp, hpp = C.POINTER(pop_config), C.POINTER(pop_hparams)
    sig = {
        "pop_workspace_bytes": (i64, [cfgp]),
        "pop_net_size": (i64, [cfgp, i32]),
        "pop_create": (C.c_int, [C.POINTER(vp), cfgp, hpp, u64, vp, i64, vp]),
        "pop_insert": (C.c_int, [vp, i32, i64, fp, fp, fp, fp, fp, i32]),
        "pop_update": (C.c_int, [vp, i32]),
        "pop_update_timed": (C.c_int, [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "pop_act": (C.c_int, [vp, fp, i32, fp, i32]),
        "pop_act_explore": (C.c_int, [vp, fp, i32, fp, i32, fp, C.c_uint32]),
        "pop_act_explore_noalloc": (C.c_int, [vp, fp, i32, fp, fp, C.c_uint32]),
        "pop_get_params": (i64, [vp, i32, i32, fp, i64, i32]),
        "pop_set_params": (C.c_int, [vp, i32, i32, fp, i64, i32]),
        "pop_copy_agent": (C.c_int, [vp, i32, i32, i32]),
        "pop_set_hparams": (C.c_int, [vp, i32, hpp]),
        "pop_set_debug": (C.c_int, [vp, i32]),
        "pop_debug_get": (i64, [vp, i32, vp, i64, i32]),
        "pop_debug_indices": (C.c_int, [vp, vp]),
        "pop_step_count": (i64, [vp]),
        "pop_buffer_count": (i64, [vp, i32]),
        "pop_sync": (C.c_int, [vp]),
        "pop_set_option": (C.c_int, [vp, i32, i64]),
        "pop_get_tuning": (C.c_int, [vp, C.POINTER(pop_tuning)]),
        "pop_destroy": (C.c_int, [vp]),
        "pop_last_error": (C.c_char_p, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _LIB = lib
    return lib


def make_config(P, obs_dim, act_dim, hidden=(256, 256), batch=256, capacity=10000, algo=POP_ALGO_TD3,
                launch=POP_LAUNCH_AUTO, rows=None, rows_critic1=0, half_tiles=0, actor_ahead=0):
    """rows: None (the library chooses), one value for all three chains, or (target, critic, actor); launch,
    rows_critic1, half_tiles, actor_ahead: the fields of pop_tuning."""
    cfg = pop_config()
    cfg.algo, cfg.P, cfg.obs_dim, cfg.act_dim = algo, P, obs_dim, act_dim
    cfg.n_hidden = len(hidden)
    for i in range(4):
        cfg.hidden[i] = hidden[i] if i < len(hidden) else 0
    cfg.batch, cfg.capacity = batch, capacity
    cfg.tuning.launch = launch
    if rows is not None:
        rt, rc, ra = (rows, rows, rows) if isinstance(rows, int) else rows
        cfg.tuning.rows_target, cfg.tuning.rows_critic, cfg.tuning.rows_actor = rt, rc, ra
    cfg.tuning.rows_critic1, cfg.tuning.half_tiles, cfg.tuning.actor_ahead = rows_critic1, half_tiles, actor_ahead
    return cfg


def make_hparams(dicts):
    """List of plain dicts (see workloads.hparams) -> ctypes array."""
    arr = (pop_hparams * len(dicts))()
    for h, dct in zip(arr, dicts):
        for name, _ in pop_hparams._fields_:
            if name in dct:
                setattr(h, name, dct[name])
    return arr


def _ptr(x, on_device):
    """Address of a torch tensor (device or host) or of a numpy array (host)."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        assert x.is_contiguous()
        assert bool(x.is_cuda) == bool(on_device)
        return C.c_void_p(x.data_ptr())
    assert not on_device and isinstance(x, np.ndarray) and x.flags["C_CONTIGUOUS"]
    return C.c_void_p(x.ctypes.data)


def _is_device(x):
    return hasattr(x, "is_cuda") and x.is_cuda


def _check(rc, ctx=None):
    if rc < 0:
        raise PopError(rc, pop_last_error(ctx))
    return rc


def pop_last_error(ctx=None):
    msg = load_library().pop_last_error(ctx)
    return msg.decode() if msg else ""


def pop_workspace_bytes(cfg):
    return _check(load_library().pop_workspace_bytes(C.byref(cfg)))


def pop_net_size(cfg, which):
    return _check(load_library().pop_net_size(C.byref(cfg), which))


def pop_create(cfg, hp, seed, workspace_ptr, workspace_bytes, stream_ptr):
    ctx = C.c_void_p()
    rc = load_library().pop_create(C.byref(ctx), C.byref(cfg), hp, seed, C.c_void_p(workspace_ptr),
                                   workspace_bytes, C.c_void_p(stream_ptr))
    _check(rc)
    return ctx


def pop_insert(ctx, agent, n, obs, act, rew, done, next_obs):
    dev = _is_device(obs)
    return _check(load_library().pop_insert(ctx, agent, n, _ptr(obs, dev), _ptr(act, dev), _ptr(rew, dev),
                                            _ptr(done, dev), _ptr(next_obs, dev), int(dev)), ctx)


def pop_update(ctx, n_steps):
    return _check(load_library().pop_update(ctx, n_steps), ctx)


KERNEL_NAMES = ("gather", "target", "critic", "wgrad_critic", "actor", "wgrad_actor", "target_critic", "step", "step_tail")


def pop_update_timed(ctx, n_steps):
    """Returns ({kernel: summed ms}, {kernel: launches})."""
    ms = (C.c_double * len(KERNEL_NAMES))()
    cnt = (C.c_int64 * len(KERNEL_NAMES))()
    _check(load_library().pop_update_timed(ctx, n_steps, ms, cnt), ctx)
    return dict(zip(KERNEL_NAMES, list(ms))), dict(zip(KERNEL_NAMES, list(cnt)))


def pop_act(ctx, obs, n, act_out):
    dev = _is_device(obs)
    return _check(load_library().pop_act(ctx, _ptr(obs, dev), n, _ptr(act_out, dev), int(dev)), ctx)


def pop_act_explore(ctx, obs, n, act_out, sigma, step):
    dev = _is_device(obs)
    sigma = np.ascontiguousarray(sigma, dtype=np.float32)
    return _check(load_library().pop_act_explore(ctx, _ptr(obs, dev), n, _ptr(act_out, dev), int(dev),
                                                 C.c_void_p(sigma.ctypes.data), int(step)), ctx)


def pop_act_explore_noalloc(ctx, obs, n, act_out, sigma, step):
    """obs and act_out: device tensors; sigma: host values, one per agent."""
    sigma = np.ascontiguousarray(sigma, dtype=np.float32)
    return _check(load_library().pop_act_explore_noalloc(ctx, _ptr(obs, True), n, _ptr(act_out, True),
                                                         C.c_void_p(sigma.ctypes.data), int(step)), ctx)


def pop_get_params(ctx, agent, which, out):
    dev = _is_device(out)
    n = out.numel() if hasattr(out, "numel") else out.size
    return _check(load_library().pop_get_params(ctx, agent, which, _ptr(out, dev), n, int(dev)), ctx)


def pop_set_params(ctx, agent, which, data):
    dev = _is_device(data)
    n = data.numel() if hasattr(data, "numel") else data.size
    return _check(load_library().pop_set_params(ctx, agent, which, _ptr(data, dev), n, int(dev)), ctx)


def pop_copy_agent(ctx, dst, src, with_buffer):
    return _check(load_library().pop_copy_agent(ctx, dst, src, int(bool(with_buffer))), ctx)


def pop_set_hparams(ctx, agent, hp):
    """hp: a plain dict (see workloads.hparams) or a pop_hparams."""
    if isinstance(hp, dict):
        hp = make_hparams([hp])[0]
    return _check(load_library().pop_set_hparams(ctx, agent, C.byref(hp)), ctx)


def pop_set_debug(ctx, on):
    return _check(load_library().pop_set_debug(ctx, int(on)), ctx)


def pop_debug_get(ctx, what, out):
    dev = _is_device(out)
    nbytes = out.numel() * out.element_size() if hasattr(out, "numel") else out.nbytes
    return _check(load_library().pop_debug_get(ctx, what, _ptr(out, dev), nbytes, int(dev)), ctx)


def pop_debug_indices(ctx, out):
    assert out.dtype == np.int64 and out.flags["C_CONTIGUOUS"]
    return _check(load_library().pop_debug_indices(ctx, C.c_void_p(out.ctypes.data)), ctx)


def pop_step_count(ctx):
    return _check(load_library().pop_step_count(ctx), ctx)


def pop_buffer_count(ctx, agent):
    return _check(load_library().pop_buffer_count(ctx, agent), ctx)


def pop_sync(ctx):
    return _check(load_library().pop_sync(ctx), ctx)


def pop_set_option(ctx, key, value):
    return _check(load_library().pop_set_option(ctx, int(key), int(value)), ctx)


def pop_get_tuning(ctx):
    """The tuning in force as a dict (field names of pop_tuning)."""
    t = pop_tuning()
    _check(load_library().pop_get_tuning(ctx, C.byref(t)), ctx)
    return {name: int(getattr(t, name)) for name, _ in pop_tuning._fields_}


def pop_destroy(ctx):
    return _check(load_library().pop_destroy(ctx))


class Population:
    """Convenience owner of one context: allocates the workspace with PyTorch on
    the given device and forwards every call to the C functions above."""

    def __init__(self, cfg, hparam_dicts, seed=0, device="cuda:0", stream=None):
        import torch
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = pop_workspace_bytes(cfg)
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            self._hp = make_hparams(hparam_dicts)
            self.ctx = pop_create(cfg, self._hp, seed, self.workspace.data_ptr(), nbytes, self.stream.cuda_stream)
        self.actor_size = pop_net_size(cfg, PARAM_CODES["actor"])
        self.critic_size = pop_net_size(cfg, PARAM_CODES["critic1"])

    def insert(self, agent, obs, act, rew, done, next_obs):
        n = rew.shape[-1]
        return pop_insert(self.ctx, agent, n, obs, act, rew, done, next_obs)

    def update(self, n_steps):
        return pop_update(self.ctx, n_steps)

    def update_timed(self, n_steps):
        return pop_update_timed(self.ctx, n_steps)

    def sync(self):
        return pop_sync(self.ctx)

    def act(self, obs, sigma=None, step=0):
        import torch
        n = obs.shape[1]
        if _is_device(obs):
            out = torch.empty((self.cfg.P, n, self.cfg.act_dim), dtype=torch.float32, device=obs.device)
        else:
            out = np.empty((self.cfg.P, n, self.cfg.act_dim), dtype=np.float32)
        if sigma is None:
            pop_act(self.ctx, obs, n, out)
        else:
            assert len(sigma) == self.cfg.P
            pop_act_explore(self.ctx, obs, n, out, sigma, step)
        return out

    def get_params(self, agent, which):
        code = PARAM_CODES[which] if isinstance(which, str) else which
        size = 1 if code >= 15 else (self.actor_size if code % 3 == 0 else self.critic_size)
        out = np.empty(size, dtype=np.float32)
        pop_get_params(self.ctx, agent, code, out)
        return out

    def set_params(self, agent, which, data):
        code = PARAM_CODES[which] if isinstance(which, str) else which
        if not _is_device(data):
            data = np.ascontiguousarray(data, dtype=np.float32)
        return pop_set_params(self.ctx, agent, code, data)

    def copy_agent(self, dst, src, with_buffer):
        return pop_copy_agent(self.ctx, dst, src, with_buffer)

    def set_hparams(self, agent, hp):
        return pop_set_hparams(self.ctx, agent, hp)

    def set_debug(self, on):
        return pop_set_debug(self.ctx, on)

    def debug(self, what):
        c, P, B = self.cfg, self.cfg.P, self.cfg.batch
        shapes = {"indices": ((P, B), np.uint32), "batch": ((P, B, 2 * c.obs_dim + c.act_dim + 2), np.float32),
                  "target_action": ((P, B, c.act_dim), np.float32), "target_y": ((P, B), np.float32),
                  "losses": ((P, 2), np.float32)}
        shape, dt = shapes[what]
        out = np.empty(shape, dtype=dt)
        pop_debug_get(self.ctx, DEBUG_CODES[what], out)
        return out

    def set_option(self, key, value):
        return pop_set_option(self.ctx, key, value)

    def tuning(self):
        return pop_get_tuning(self.ctx)

    def step_count(self):
        return pop_step_count(self.ctx)

    def buffer_count(self, agent):
        return pop_buffer_count(self.ctx, agent)

    def close(self):
        if self.ctx is not None:
            pop_sync(self.ctx)
            pop_destroy(self.ctx)
            self.ctx = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
