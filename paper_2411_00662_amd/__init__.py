"""MI355X-native MoE token dispatch / combine path of MoNTA (arxiv 2411.00662).

The product is ``libmonta.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/monta.h``); this package is its thin ctypes binding plus device-buffer
plumbing.  Build with ``python -m paper_2411_00662_amd.build``.
"""
from .binding import (BF16, FP32, MontaError, make_cfg, monta_cfg, monta_ws_layout, monta_workspace_bytes,
                      monta_ws_layout_query, monta_ws_init, monta_gate, monta_expert_linear, monta_route_dispatch_expert, monta_route, monta_dispatch, monta_regather,
                      monta_dispatch_regather, monta_route_dispatch_regather, monta_combine, monta_unregather, monta_combine_staged,
                      monta_unregather_combine, monta_allgather, monta_allgather_regather, monta_set_pipeline_mode, monta_get_pipeline_mode, monta_pipeline_query, monta_set_cache_policy, monta_get_cache_policy, monta_set_plan_mode, monta_get_plan_mode,
                      monta_copy, monta_profile_enable, monta_profile_reset, monta_profile_read, monta_strerror,
                      monta_last_hip_error, monta_shutdown, monta_route_dispatch_combine_static, make_plan_in, monta_plan_chunk_times, monta_plan_strategy, monta_plan_in,
                      monta_plan_out, monta_curve, KERNEL_NAMES, EXPORTS, LIB_PATH)
from .buffers import Buffers, alloc_buffers, read_tables

__all__ = [n for n in dir() if not n.startswith("_")]
