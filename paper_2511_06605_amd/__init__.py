"""MI355X copy collectives (all-gather, all-to-all, broadcast, batched
back-to-back copies) executed by hand-written HIP kernels behind a C boundary.

``binding`` mirrors ``include/dmalatte.h``; ``inputs`` draws seeded synthetic
workloads; ``build`` compiles the library in-tree.  Nothing here computes a
result on the CPU.
"""

from .binding import (  # noqa: F401
    DL_ERR_EXPIRED, DL_ERR_LOST, DL_ERR_CAPACITY, DL_STATIC_MAX_COPIES, DL_DISPATCH_DEVICE_MAX_TOKENS, DL_ERR_HIP, DL_ERR_INVALID, DL_ERR_OVERLAP, DL_ERR_STATE, DL_ERR_TIMEOUT, DL_MAX_FANOUT,
    DL_MODE_ONESHOT, DL_MODE_PRELAUNCH, DL_MODE_SIGNAL, DL_MODE_STANDBY, DL_MODE_AUTO, DL_OK, DL_OP_BATCH, DL_OP_BROADCAST, DL_OP_ALLGATHER, DL_OP_ALLTOALL, DL_OP_SWAP,
    DL_OP_TOKEN_DISPATCH, DL_AUTO_STANDBY_TILES, DL_AUTO_SIGNAL_MAX_BYTES, DL_AUTO_PRELAUNCH_MAX_BYTES, DL_PLAN_FANOUT, Config, DlError, dl_allgather,
    dl_alltoall, dl_batch_copy, dl_broadcast, dl_get_config, dl_get_mode, dl_init, dl_last_ticket,
    dl_plan_allgather, dl_plan_alltoall, dl_plan_batch, dl_plan_broadcast, dl_plan_first_hazard,
    dl_plan_tiles, dl_prelaunch_start, dl_prelaunch_stop, dl_set_config, dl_set_mode,
    dl_set_validate, dl_shutdown, dl_trigger, dl_wait, dl_wait_armed, dl_batch_swap, dl_alltoall_inplace,
    dl_plan_alltoall_inplace, dl_plan_swap_first_hazard, dl_batch_fanout, dl_token_dispatch,
    dl_plan_token_dispatch, dl_plan_batch_inferred, dl_set_trace, dl_get_trace, dl_trace_clock,
    dl_last_device_error, dl_debug_lose_next_table, dl_batch_copy_static, dl_plan_mode, dl_last_mode,
    dl_complete, dl_parse_config, dl_token_dispatch_device)
