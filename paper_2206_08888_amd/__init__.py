"""MI355X-native population TD3 update engine (C-ABI HIP library + thin binding).

The computation lives entirely in libpop.so (hand-written gfx950 kernels);
this package only marshals arguments.  PyTorch is used by callers to allocate
the device workspace and to supply a stream.
"""
from .binding import (  # noqa: F401
    POP_ALGO_SAC, POP_ALGO_TD3, POP_ALGO_TD3_SHARED, POP_LAUNCH_AUTO, POP_LAUNCH_PER_PART, POP_LAUNCH_SINGLE, POP_LAUNCH_TAIL,
    POP_LAUNCH_TARGET_CRITIC, POP_OPT_WAIT_LIMIT_TICKS, POP_EEMPTY, POP_EHIP, POP_EINVAL, POP_ENOMEM, POP_EUNSUPPORTED, POP_OK,
    PARAM_CODES, DEBUG_CODES, PopError, Population, lib_path, load_library, make_config, make_hparams,
    pop_act, pop_act_explore, pop_act_explore_noalloc, pop_buffer_count, pop_create, pop_debug_get, pop_debug_indices, pop_destroy, pop_get_params,
    pop_insert, pop_last_error, pop_net_size, pop_copy_agent, pop_set_debug, pop_set_hparams, pop_set_option, pop_get_tuning, pop_set_params, pop_step_count, pop_sync, pop_update, pop_update_timed, KERNEL_NAMES,
    pop_workspace_bytes, pop_config, pop_hparams, pop_tuning,
)
