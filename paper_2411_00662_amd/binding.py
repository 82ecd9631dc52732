"""ctypes binding of the C ABI in include/monta.h.

Argument marshalling only: every function here has the name and the argument
order of its C counterpart, turns torch tensors into raw device pointers, checks
that the tensors are large enough for the shapes in ``cfg`` (the C side sees
only pointers), and raises ``MontaError`` on a negative status.  No step of the
path runs in Python, and there is no fallback: if ``libmonta.so`` has not been
built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmonta.so")

FP32, BF16 = 0, 1
(K_ROUTE, K_POSITIONS, K_PACK, K_REGATHER, K_PACK_REGATHER, K_COMBINE, K_COPY, K_PLAN_PACK, K_UNREGATHER,
 K_UNREGATHER_COMBINE, K_ALLGATHER, K_GATE, K_EXPERT) = range(13)
KERNEL_NAMES = ["route_plan", "positions", "pack", "regather", "pack_regather", "combine", "copy", "plan_pack",
                "unregather", "unregather_combine", "allgather", "gate", "expert", "allgather_regather"]


class MontaError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str = ""):
        self.code = code
        super().__init__(f"{what}: {detail} (status {code})")


class monta_cfg(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64), ("hidden", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("experts", ctypes.c_int32), ("top_k", ctypes.c_int32), ("ep", ctypes.c_int32),
                ("tp", ctypes.c_int32), ("slices", ctypes.c_int32), ("capacity_factor", ctypes.c_float),
                ("renorm", ctypes.c_int32), ("padded", ctypes.c_int32)]


class monta_ws_layout(ctypes.Structure):
    _fields_ = [("ws_bytes", ctypes.c_int64), ("max_rows", ctypes.c_int64), ("capacity", ctypes.c_int64),
                ("units", ctypes.c_int32), ("tokens_per_unit", ctypes.c_int32), ("block_tokens", ctypes.c_int32),
                ("num_blocks", ctypes.c_int32),
                ("off_meta", ctypes.c_int64), ("off_counts", ctypes.c_int64), ("off_kept", ctypes.c_int64),
                ("off_offsets", ctypes.c_int64), ("off_n", ctypes.c_int64), ("off_stage_off", ctypes.c_int64),
                ("off_unit_base", ctypes.c_int64), ("off_send_rows", ctypes.c_int64),
                ("off_unit_rows", ctypes.c_int64), ("off_pos_final", ctypes.c_int64),
                ("off_pos_stage", ctypes.c_int64), ("off_row_map", ctypes.c_int64),
                ("off_block_counts", ctypes.c_int64), ("off_block_base", ctypes.c_int64),
                ("off_local_rank", ctypes.c_int64),
                ("off_kept_prefix", ctypes.c_int64)]


class monta_curve(ctypes.Structure):
    _fields_ = [("volume", ctypes.POINTER(ctypes.c_double)), ("eff", ctypes.POINTER(ctypes.c_double)),
                ("n", ctypes.c_int32)]


class monta_plan_in(ctypes.Structure):
    _fields_ = [("traffic", ctypes.c_double), ("t", ctypes.c_int32), ("e", ctypes.c_int32),
                ("b1", ctypes.c_double), ("b2", ctypes.c_double), ("b3", ctypes.c_double),
                ("r1", monta_curve), ("r2", monta_curve), ("r3", monta_curve),
                ("i_minimal", ctypes.c_double), ("n_max", ctypes.c_int32)]


class monta_plan_out(ctypes.Structure):
    _fields_ = [("t_base", ctypes.c_double), ("t_o1", ctypes.c_double), ("t_o2", ctypes.c_double),
                ("t_o3", ctypes.c_double), ("n_o2", ctypes.c_int32), ("n_o3", ctypes.c_int32),
                ("strategy", ctypes.c_int32), ("chunks", ctypes.c_int32), ("t_best", ctypes.c_double)]


# every symbol include/monta.h declares
EXPORTS = ["monta_workspace_bytes", "monta_ws_layout_query", "monta_ws_init", "monta_gate", "monta_expert_linear", "monta_route_dispatch_expert", "monta_route", "monta_dispatch",
           "monta_regather", "monta_dispatch_regather", "monta_route_dispatch_regather", "monta_combine", "monta_unregather", "monta_combine_staged",
           "monta_unregather_combine", "monta_allgather", "monta_set_pipeline_mode",
           "monta_get_pipeline_mode", "monta_set_plan_mode", "monta_get_plan_mode", "monta_set_cache_policy", "monta_get_cache_policy", "monta_copy", "monta_profile_enable", "monta_profile_reset",
           "monta_profile_read", "monta_plan_chunk_times", "monta_plan_strategy", "monta_strerror",
           "monta_last_hip_error", "monta_shutdown", "monta_route_dispatch_combine_static", "monta_pipeline_query", "monta_allgather_regather"]

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2411_00662_amd.build); "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64p = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)
        cfgp = ctypes.POINTER(monta_cfg)
        L.monta_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t), i64p]
        L.monta_ws_layout_query.argtypes = [cfgp, ctypes.POINTER(monta_ws_layout)]
        L.monta_ws_init.argtypes = [cfgp, vp, vp]
        L.monta_route.argtypes = [cfgp, vp, vp, vp, vp, vp]
        L.monta_dispatch.argtypes = [cfgp, vp, vp, vp, i32, vp]
        L.monta_regather.argtypes = [cfgp, vp, vp, vp, i32, vp]
        L.monta_dispatch_regather.argtypes = [cfgp, vp, vp, vp, vp, vp]
        L.monta_combine.argtypes = [cfgp, vp, vp, vp, vp, vp]
        L.monta_route_dispatch_regather.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.monta_unregather.argtypes = [cfgp, vp, vp, vp, i32, vp]
        L.monta_allgather.argtypes = [cfgp, vp, vp, vp, i32, vp]
        L.monta_allgather_regather.argtypes = [cfgp, vp, vp, vp, vp, i32, vp]
        L.monta_combine_staged.argtypes = [cfgp, vp, vp, vp, vp, i32, vp]
        L.monta_unregather_combine.argtypes = [cfgp, vp, vp, vp, vp, vp, vp]
        L.monta_set_pipeline_mode.argtypes = [i32]
        L.monta_get_pipeline_mode.argtypes = []
        L.monta_set_cache_policy.argtypes = [i32]
        L.monta_set_plan_mode.argtypes = [i32]
        L.monta_get_plan_mode.argtypes = []
        L.monta_get_cache_policy.argtypes = []
        L.monta_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.monta_gate.argtypes = [ctypes.POINTER(monta_cfg), vp, vp, vp, vp]
        L.monta_expert_linear.argtypes = [ctypes.POINTER(monta_cfg), vp, vp, i32, vp, vp, i32, vp]
        L.monta_route_dispatch_expert.argtypes = [ctypes.POINTER(monta_cfg), vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i32, vp]
        L.monta_profile_enable.argtypes = [i32]
        L.monta_profile_reset.argtypes = []
        L.monta_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), i64p]
        L.monta_plan_chunk_times.argtypes = [ctypes.POINTER(monta_plan_in), i32] + [ctypes.POINTER(ctypes.c_double)] * 3
        L.monta_plan_strategy.argtypes = [ctypes.POINTER(monta_plan_in), ctypes.POINTER(monta_plan_out)]
        L.monta_strerror.argtypes = [i32]
        L.monta_strerror.restype = ctypes.c_char_p
        L.monta_last_hip_error.argtypes = []
        L.monta_shutdown.argtypes = []
        L.monta_pipeline_query.argtypes = [cfgp] + [ctypes.POINTER(ctypes.c_int32)] * 4
        L.monta_route_dispatch_combine_static.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp]
        for name in EXPORTS:
            if name != "monta_strerror":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def monta_strerror(code: int) -> str:
    return lib().monta_strerror(int(code)).decode()


def monta_last_hip_error() -> int:
    return int(lib().monta_last_hip_error())


def monta_shutdown():
    _check(lib().monta_shutdown(), "monta_shutdown")


def _check(code: int, what: str):
    if code != 0:
        detail = monta_strerror(code)
        if code == -4:
            detail += f", hipError_t {monta_last_hip_error()}"
        raise MontaError(code, what, detail)


def make_cfg(tokens, hidden, dtype, experts, top_k, ep, tp, slices, capacity_factor=0.0, renorm=1, padded=0) -> monta_cfg:
    return monta_cfg(int(tokens), int(hidden), int(dtype), int(experts), int(top_k), int(ep), int(tp), int(slices),
                     float(capacity_factor), int(renorm), int(padded))


def _bpe(cfg) -> int:
    return 4 if cfg.dtype == FP32 else 2


def _ptr(t, min_bytes: int, name: str) -> int:
    """Raw pointer of a torch tensor (or an int address, passed through unchecked)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous tensor")
    have = t.numel() * t.element_size()
    if have < min_bytes:
        raise ValueError(f"{name}: tensor holds {have} bytes, the shapes in cfg need {min_bytes}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def monta_workspace_bytes(cfg):
    ws, rows = ctypes.c_size_t(0), ctypes.c_int64(0)
    _check(lib().monta_workspace_bytes(ctypes.byref(cfg), ctypes.byref(ws), ctypes.byref(rows)), "monta_workspace_bytes")
    return int(ws.value), int(rows.value)


def monta_ws_layout_query(cfg) -> monta_ws_layout:
    L = monta_ws_layout()
    _check(lib().monta_ws_layout_query(ctypes.byref(cfg), ctypes.byref(L)), "monta_ws_layout_query")
    return L


def monta_ws_init(cfg, ws, stream=None):
    L = monta_ws_layout_query(cfg)
    _check(lib().monta_ws_init(ctypes.byref(cfg), _ptr(ws, L.ws_bytes, "ws"), _stream(stream)), "monta_ws_init")


def monta_route(cfg, logits, topk_idx, gates, ws, stream=None):
    L = monta_ws_layout_query(cfg)
    T, E, k = cfg.tokens, cfg.experts, cfg.top_k
    _check(lib().monta_route(ctypes.byref(cfg), _ptr(logits, T * E * 4, "logits"), _ptr(topk_idx, T * k * 4, "topk_idx"),
                             _ptr(gates, T * k * 4, "gates"), _ptr(ws, L.ws_bytes, "ws"), _stream(stream)),
           "monta_route")


def monta_dispatch(cfg, x, stage, ws, slice=-1, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_dispatch(ctypes.byref(cfg), _ptr(x, cfg.tokens * row, "x"), _ptr(stage, L.max_rows * row, "stage"),
                                _ptr(ws, L.ws_bytes, "ws"), int(slice), _stream(stream)), "monta_dispatch")


def monta_regather(cfg, stage, final_, ws, slice=-1, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_regather(ctypes.byref(cfg), _ptr(stage, L.max_rows * row, "stage"),
                                _ptr(final_, L.max_rows * row, "final_"), _ptr(ws, L.ws_bytes, "ws"), int(slice),
                                _stream(stream)), "monta_regather")


def monta_dispatch_regather(cfg, x, stage, final_, ws, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_dispatch_regather(ctypes.byref(cfg), _ptr(x, cfg.tokens * row, "x"),
                                         _ptr(stage, L.max_rows * row, "stage"), _ptr(final_, L.max_rows * row, "final_"),
                                         _ptr(ws, L.ws_bytes, "ws"), _stream(stream)), "monta_dispatch_regather")


def monta_route_dispatch_regather(cfg, logits, x, topk_idx, gates, stage, final_, ws, stream=None):
    L = monta_ws_layout_query(cfg)
    T, E, k = cfg.tokens, cfg.experts, cfg.top_k
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_route_dispatch_regather(
        ctypes.byref(cfg), _ptr(logits, T * E * 4, "logits"), _ptr(x, T * row, "x"), _ptr(topk_idx, T * k * 4, "topk_idx"),
        _ptr(gates, T * k * 4, "gates"), _ptr(stage, L.max_rows * row, "stage"), _ptr(final_, L.max_rows * row, "final_"),
        _ptr(ws, L.ws_bytes, "ws"), _stream(stream)), "monta_route_dispatch_regather")


def monta_route_dispatch_combine_static(cfg, logits, x, topk_idx, gates, stage, final_, out, stream=None):
    L = monta_ws_layout_query(cfg)
    T, E, k = cfg.tokens, cfg.experts, cfg.top_k
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_route_dispatch_combine_static(
        ctypes.byref(cfg), _ptr(logits, T * E * 4, "logits"), _ptr(x, T * row, "x"), _ptr(topk_idx, T * k * 4, "topk_idx"),
        _ptr(gates, T * k * 4, "gates"), _ptr(stage, L.max_rows * row, "stage"), _ptr(final_, L.max_rows * row, "final_"),
        _ptr(out, T * row, "out"), _stream(stream)), "monta_route_dispatch_combine_static")


def monta_allgather_regather(cfg, stage, gathered, final_, ws, schedule=1, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_allgather_regather(ctypes.byref(cfg), _ptr(stage, L.max_rows * row, "stage"),
                                          _ptr(gathered, L.max_rows * row, "gathered"), _ptr(final_, L.max_rows * row, "final_"),
                                          _ptr(ws, L.ws_bytes, "ws"), int(schedule), _stream(stream)), "monta_allgather_regather")


def monta_combine(cfg, y, gates, out, ws, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_combine(ctypes.byref(cfg), _ptr(y, L.max_rows * row, "y"),
                               _ptr(gates, cfg.tokens * cfg.top_k * 4, "gates"), _ptr(out, cfg.tokens * row, "out"),
                               _ptr(ws, L.ws_bytes, "ws"), _stream(stream)), "monta_combine")


def monta_allgather(cfg, stage, gathered, ws, slice=-1, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_allgather(ctypes.byref(cfg), _ptr(stage, L.max_rows * row, "stage"),
                                 _ptr(gathered, L.max_rows * row, "gathered"), _ptr(ws, L.ws_bytes, "ws"), int(slice),
                                 _stream(stream)), "monta_allgather")


def monta_unregather(cfg, y, y_stage, ws, slice=-1, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_unregather(ctypes.byref(cfg), _ptr(y, L.max_rows * row, "y"), _ptr(y_stage, L.max_rows * row, "y_stage"),
                                  _ptr(ws, L.ws_bytes, "ws"), int(slice), _stream(stream)), "monta_unregather")


def monta_combine_staged(cfg, y_stage, gates, out, ws, slice=-1, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_combine_staged(ctypes.byref(cfg), _ptr(y_stage, L.max_rows * row, "y_stage"),
                                      _ptr(gates, cfg.tokens * cfg.top_k * 4, "gates"), _ptr(out, cfg.tokens * row, "out"),
                                      _ptr(ws, L.ws_bytes, "ws"), int(slice), _stream(stream)), "monta_combine_staged")


def monta_unregather_combine(cfg, y, y_stage, gates, out, ws, stream=None):
    L = monta_ws_layout_query(cfg)
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_unregather_combine(ctypes.byref(cfg), _ptr(y, L.max_rows * row, "y"),
                                          _ptr(y_stage, L.max_rows * row, "y_stage"),
                                          _ptr(gates, cfg.tokens * cfg.top_k * 4, "gates"), _ptr(out, cfg.tokens * row, "out"),
                                          _ptr(ws, L.ws_bytes, "ws"), _stream(stream)), "monta_unregather_combine")


def monta_set_pipeline_mode(mode: int):
    _check(lib().monta_set_pipeline_mode(int(mode)), "monta_set_pipeline_mode")


def monta_get_pipeline_mode() -> int:
    return int(lib().monta_get_pipeline_mode())


def monta_pipeline_query(cfg):
    """-> (mode, slices of the first launch, slices per later launch, plan fused with the first pack)."""
    a, f, b, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().monta_pipeline_query(ctypes.byref(cfg), ctypes.byref(a), ctypes.byref(f), ctypes.byref(b), ctypes.byref(c)),
           "monta_pipeline_query")
    return a.value, f.value, b.value, bool(c.value)


def monta_set_plan_mode(mode: int):
    _check(lib().monta_set_plan_mode(int(mode)), "monta_set_plan_mode")


def monta_get_plan_mode() -> int:
    return int(lib().monta_get_plan_mode())


def monta_set_cache_policy(policy: int):
    _check(lib().monta_set_cache_policy(int(policy)), "monta_set_cache_policy")


def monta_get_cache_policy() -> int:
    return int(lib().monta_get_cache_policy())


def monta_gate(cfg, x, w_gate, logits, stream=None):
    row = cfg.hidden * _bpe(cfg)
    _check(lib().monta_gate(ctypes.byref(cfg), _ptr(x, cfg.tokens * row, "x"), _ptr(w_gate, cfg.experts * row, "w_gate"),
                            _ptr(logits, cfg.tokens * cfg.experts * 4, "logits"), _stream(stream)), "monta_gate")


def monta_expert_linear(cfg, x_final, w_exp, out_features: int, y, ws, slice: int = -1, stream=None):
    L = monta_ws_layout_query(cfg)
    bpe = _bpe(cfg)
    _check(lib().monta_expert_linear(ctypes.byref(cfg), _ptr(x_final, L.max_rows * cfg.hidden * bpe, "x_final"),
                                     _ptr(w_exp, cfg.experts * int(out_features) * cfg.hidden * bpe, "w_exp"),
                                     int(out_features), _ptr(y, L.max_rows * int(out_features) * bpe, "y"),
                                     _ptr(ws, L.ws_bytes, "ws"), int(slice), _stream(stream)), "monta_expert_linear")


def monta_route_dispatch_expert(cfg, logits, x, topk_idx, gates, stage, final, w_exp, out_features: int, y, ws,
                                overlap: int = 1, stream=None):
    L = monta_ws_layout_query(cfg)
    bpe = _bpe(cfg)
    row = cfg.hidden * bpe
    T, k = cfg.tokens, cfg.top_k
    _check(lib().monta_route_dispatch_expert(
        ctypes.byref(cfg), _ptr(logits, T * cfg.experts * 4, "logits"), _ptr(x, T * row, "x"),
        _ptr(topk_idx, T * k * 4, "topk_idx"), _ptr(gates, T * k * 4, "gates"), _ptr(stage, L.max_rows * row, "stage"),
        _ptr(final, L.max_rows * row, "final"), _ptr(w_exp, cfg.experts * int(out_features) * row, "w_exp"),
        int(out_features), _ptr(y, L.max_rows * int(out_features) * bpe, "y"), _ptr(ws, L.ws_bytes, "ws"), int(overlap),
        _stream(stream)), "monta_route_dispatch_expert")


def monta_copy(dst, src, nbytes: int, stream=None):
    _check(lib().monta_copy(_ptr(dst, nbytes, "dst"), _ptr(src, nbytes, "src"), int(nbytes), _stream(stream)), "monta_copy")


def monta_profile_enable(on: bool):
    _check(lib().monta_profile_enable(1 if on else 0), "monta_profile_enable")


def monta_profile_reset():
    _check(lib().monta_profile_reset(), "monta_profile_reset")


def monta_profile_read(kernel_id: int):
    ms, n = ctypes.c_double(0), ctypes.c_int64(0)
    _check(lib().monta_profile_read(int(kernel_id), ctypes.byref(ms), ctypes.byref(n)), "monta_profile_read")
    return float(ms.value), int(n.value)


def _curve(points):
    """[(volume_bytes, efficiency), ...] -> (monta_curve, keep-alive arrays)."""
    n = len(points)
    vol = (ctypes.c_double * n)(*[float(p[0]) for p in points])
    eff = (ctypes.c_double * n)(*[float(p[1]) for p in points])
    return monta_curve(ctypes.cast(vol, ctypes.POINTER(ctypes.c_double)), ctypes.cast(eff, ctypes.POINTER(ctypes.c_double)), n), (vol, eff)


def make_plan_in(traffic, t, e, b1, b2, b3, r1, r2, r3, i_minimal, n_max=1 << 16):
    """Curves are lists of (volume in bytes, efficiency).  Returns (monta_plan_in, keep-alive tuple)."""
    c1, k1 = _curve(r1)
    c2, k2 = _curve(r2)
    c3, k3 = _curve(r3)
    return monta_plan_in(float(traffic), int(t), int(e), float(b1), float(b2), float(b3), c1, c2, c3,
                         float(i_minimal), int(n_max)), (k1, k2, k3)


def monta_plan_chunk_times(pin, n: int):
    aa, ag, d2d = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().monta_plan_chunk_times(ctypes.byref(pin), int(n), ctypes.byref(aa), ctypes.byref(ag), ctypes.byref(d2d)),
           "monta_plan_chunk_times")
    return aa.value, ag.value, d2d.value


def monta_plan_strategy(pin) -> monta_plan_out:
    out = monta_plan_out()
    _check(lib().monta_plan_strategy(ctypes.byref(pin), ctypes.byref(out)), "monta_plan_strategy")
    return out
