"""Slow Momentum (Algorithm 1 of the paper) hot path for one MI355X:
hand-written gfx950 kernels behind a C ABI (include/slowmo.h), with a ctypes
binding of the same names (binding.py) and a small PyTorch-facing holder
(optimizer.py).  The compiled library is required; nothing falls back to CPU.
"""
from . import binding  # noqa: F401
from .binding import (SlowMoError, slowmo_config, slowmo_create, slowmo_destroy,  # noqa: F401
                      slowmo_get_buffer, slowmo_get_counters, slowmo_last_error,
                      slowmo_expgraph_in_peers, slowmo_export_bytes, slowmo_export_state,
                      slowmo_import_state, slowmo_local_outer_step, slowmo_local_step,
                      slowmo_mix_step, slowmo_local_mix_step, slowmo_plan_mix, slowmo_check_device_range, slowmo_get_pushsum_weights, slowmo_debias,
                      slowmo_debias_static, slowmo_lr_step_decay, slowmo_lr_inverse_sqrt,
                      slowmo_set_tensor_hparams,
                      slowmo_outer_step, slowmo_plan_local,
                      slowmo_plan_outer, slowmo_state_bytes, slowmo_version)


def __getattr__(name):          # torch is imported only when the holder is used
    if name in ("SlowMo", "make_config"):
        from . import optimizer
        return getattr(optimizer, name)
    raise AttributeError(name)
