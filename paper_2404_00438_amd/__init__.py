"""Distributed Lion optimizer sweep for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

``binding`` exposes the entry points of ``include/dlion.h`` under the same
names; it marshals torch tensors into pointers and strides and nothing else.
``workloads`` holds the seeded synthetic input recipes (no arithmetic of the
method).  The library is loaded on first use and the load fails loudly if
``libdlion.so`` has not been built -- there is no fallback path.
"""
from .binding import (  # noqa: F401
    AVG,
    VOTE,
    DlionError,
    SegTable,
    dlion_aggregate,
    dlion_aggregate_encode,
    dlion_apply_encoded,
    dlion_delta_planes,
    dlion_global_lion_step,
    dlion_step_pw,
    dlion_worker_step_pw,
    dlion_aggregate_apply,
    dlion_aggregate_apply_mt,
    dlion_aggregate_mt,
    dlion_apply,
    dlion_apply_mt,
    dlion_step,
    dlion_step_mt,
    dlion_step_mt_workspace_bytes,
    dlion_get_tuning,
    dlion_membench,
    dlion_noalloc_init,
    dlion_step_noalloc,
    dlion_set_tuning,
    tuned,
    Tuning,
    dlion_step_workspace_bytes,
    dlion_step_ws,
    dlion_version,
    dlion_worker_step,
    dlion_worker_step_mt,
    load_library,
    words_for,
)
