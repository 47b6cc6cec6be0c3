"""MI355X-native hot path of CoCoD-SGD: one round of Algorithm 1 for W simulated workers on one GPU.

`binding` is a thin ctypes layer over libcocod.so (hand-written HIP for gfx950); it only marshals
arguments.  Build the library with `python -m paper_1906_12043_amd.build`.
"""
from .binding import (  # noqa: F401
    CocodError, Config, Context, lib, lib_path, plan_layout, debug_normals, debug_copy,
    cocod_create, cocod_destroy, cocod_local_steps, cocod_average_begin, cocod_average_end_apply,
    GRAD_QUADRATIC, GRAD_MLP, GRAD_EXTERNAL, SCHED_OVERLAP, SCHED_SERIAL, SCHED_FUSED, SCHED_HEAD, FLAG_DRY_RUN,
    OK, ERR_INVALID, ERR_STATE, ERR_HIP, ERR_NOMEM, ERR_UNSUPPORTED,
)
