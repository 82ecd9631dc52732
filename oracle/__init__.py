"""ctypes front end of the plain-C CPU oracle (``monta_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg use it; the product package never imports it, and it never
imports the product package.  The C file is compiled with plain ``gcc`` (no HIP).

All functions take and return numpy arrays.  bf16 activations travel as
``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "monta_oracle.c")
_LIB = os.path.join(_HERE, "libmonta_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libmonta_oracle_omp.so")     # same source with -fopenmp: the all-cores timing build
_libs = {}
_use_omp = False


def build(force: bool = False) -> str:
    """Compile the oracle with gcc, twice: the plain single-threaded build (the parity reference) and the same
    source with -fopenmp (the all-cores CPU baseline).  -O1 and no fast-math: keep it plain and IEEE."""
    for lib, extra in ((_LIB, []), (_LIB_OMP, ["-fopenmp"])):
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
            cmd = ["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fno-fast-math",
                   "-ffp-contract=off", "-Wall", "-Wextra", *extra, "-o", lib, _SRC, "-lm"]
            subprocess.run(cmd, check=True)
    return _LIB


class all_cores:
    """``with oracle.all_cores():`` routes the calls inside to the OpenMP build (timing only)."""

    def __enter__(self):
        global _use_omp
        self._old = _use_omp
        _use_omp = True
        return self

    def __exit__(self, *exc):
        global _use_omp
        _use_omp = self._old


def threads() -> int:
    """Threads the current build's loops run on (1 for the plain build)."""
    return int(_load().monta_oracle_threads())


def _load():
    path = _LIB_OMP if _use_omp else _LIB
    lib = _libs.get(path)
    if lib is None:
        build()
        lib = ctypes.CDLL(path)
        lib.monta_oracle_capacity.restype = ctypes.c_int64
        lib.monta_oracle_capacity.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        _libs[path] = lib
    return lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: error {rc}")


def capacity(T: int, E: int, k: int, cf: float) -> int:
    return int(_load().monta_oracle_capacity(T, E, k, float(cf)))


def route(logits: np.ndarray, k: int, renorm: int = 1):
    """logits float32 [T,E] -> (topk_idx int32 [T,k], gates float32 [T,k])."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    if not np.isfinite(logits).all():
        raise ValueError("oracle route: logits must be finite")
    T, E = logits.shape
    idx = np.empty((T, k), np.int32)
    gates = np.empty((T, k), np.float32)
    rc = _load().monta_oracle_route(ctypes.c_int64(T), E, k, int(renorm), _p(logits), _p(idx), _p(gates))
    _check(rc, "route")
    return idx, gates


def gate(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Gate projection: x [T,H], w [E,H] (float32, or uint16 bf16 bits) -> logits float32 [T,E]."""
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    if x.dtype != w.dtype or x.dtype not in (np.float32, np.uint16) or x.shape[1] != w.shape[1]:
        raise ValueError("oracle gate: x and w must share dtype (float32 or uint16) and hidden size")
    T, H = x.shape
    E = w.shape[0]
    logits = np.empty((T, E), np.float32)
    rc = _load().monta_oracle_gate(ctypes.c_int64(T), H, E, 0 if x.dtype == np.float32 else 1, _p(x), _p(w), _p(logits))
    _check(rc, "gate")
    return logits


@dataclass
class Plan:
    C: int
    R: int                  # kept pairs = STAGE rows
    final_rows: int         # rows of FINAL: R (compact) or E*C (padded)
    alive: int
    counts: np.ndarray      # [E]
    kept: np.ndarray        # [E]
    offsets: np.ndarray     # [E+1]
    pos_final: np.ndarray   # [T,k]
    n: np.ndarray           # [U,E]
    stage_off: np.ndarray   # [U,E]
    unit_base: np.ndarray   # [U,E]
    pos_stage: np.ndarray   # [T,k]
    send_rows: np.ndarray   # [U,ep]


def plan(topk_idx: np.ndarray, E: int, ep: int, tp: int, S: int, cf: float, padded: int = 0) -> Plan:
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, k = topk_idx.shape
    U = S * tp
    counts = np.empty(E, np.int32)
    kept = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    pos_final = np.empty((T, k), np.int32)
    n = np.empty((U, E), np.int32)
    stage_off = np.empty((U, E), np.int32)
    unit_base = np.empty((U, E), np.int32)
    pos_stage = np.empty((T, k), np.int32)
    send_rows = np.empty((U, ep), np.int32)
    alive = ctypes.c_int64(0)
    kept_rows = ctypes.c_int64(0)
    rc = _load().monta_oracle_plan(ctypes.c_int64(T), E, k, ep, tp, S, ctypes.c_double(cf), int(padded),
                                   ctypes.byref(kept_rows), _p(topk_idx),
                                   _p(counts), _p(kept), _p(offsets), _p(pos_final), _p(n), _p(stage_off),
                                   _p(unit_base), _p(pos_stage), _p(send_rows), ctypes.byref(alive))
    _check(rc, "plan")
    return Plan(capacity(T, E, k, cf), int(kept_rows.value), int(offsets[E]), int(alive.value), counts, kept, offsets,
                pos_final, n, stage_off, unit_base, pos_stage, send_rows)


def pack(x: np.ndarray, pl: Plan, tp: int, S: int, stage: np.ndarray | None = None, slice_: int = -1,
         fill: int = 0) -> np.ndarray:
    """x [T,H] (float32 or uint16) -> STAGE [R,H].  Rows are bit copies."""
    x = np.ascontiguousarray(x)
    T, H = x.shape
    k = pl.pos_stage.shape[1]
    if stage is None:
        stage = np.full((pl.R, H), fill, dtype=x.dtype)
    rc = _load().monta_oracle_pack(ctypes.c_int64(T), k, tp, S, ctypes.c_int64(H * x.itemsize), _p(x),
                                   _p(pl.pos_stage), _p(stage), slice_)
    _check(rc, "pack")
    return stage


def regather(stage: np.ndarray, pl: Plan, tp: int, S: int, final: np.ndarray | None = None,
             slice_: int = -1, fill: int = 0) -> np.ndarray:
    stage = np.ascontiguousarray(stage)
    H = stage.shape[1]
    E = pl.counts.shape[0]
    if final is None:
        final = np.full((pl.final_rows, H), fill, dtype=stage.dtype)
    rc = _load().monta_oracle_regather(tp, S, E, ctypes.c_int64(H * stage.itemsize), _p(pl.n), _p(pl.stage_off),
                                       _p(pl.unit_base), _p(stage), _p(final), slice_)
    _check(rc, "regather")
    return final


def allgather(stage: np.ndarray, pl: Plan, tp: int, S: int, gathered: np.ndarray | None = None, slice_: int = -1,
              fill: int = 0) -> np.ndarray:
    """The gather as a pass of its own: the slice's STAGE range, unchanged, in a second buffer."""
    stage = np.ascontiguousarray(stage)
    H = stage.shape[1]
    E = pl.counts.shape[0]
    if gathered is None:
        gathered = np.full((pl.R, H), fill, dtype=stage.dtype)
    rc = _load().monta_oracle_allgather(tp, S, E, ctypes.c_int64(H * stage.itemsize), _p(pl.n), _p(pl.stage_off),
                                        _p(stage), _p(gathered), slice_)
    _check(rc, "allgather")
    return gathered


def pad(final: np.ndarray, pl: Plan) -> np.ndarray:
    """Zero-fills the padding rows of the capacity-padded layout (no-op for the compact layout)."""
    E = pl.counts.shape[0]
    rc = _load().monta_oracle_pad(E, ctypes.c_int64(final.shape[1] * final.itemsize), _p(pl.kept), _p(pl.offsets), _p(final))
    _check(rc, "pad")
    return final


def combine(y: np.ndarray, gates: np.ndarray, pos_final: np.ndarray, out: np.ndarray | None = None) -> np.ndarray:
    """y [R,H] float32 or uint16(bf16) -> out [T,H] of the same type (a preallocated `out` is filled in place)."""
    y = np.ascontiguousarray(y)
    gates = np.ascontiguousarray(gates, dtype=np.float32)
    pos_final = np.ascontiguousarray(pos_final, dtype=np.int32)
    T, k = pos_final.shape
    H = y.shape[1]
    if y.dtype == np.float32:
        dtype = 0
    elif y.dtype == np.uint16:
        dtype = 1
    else:
        raise ValueError("oracle combine: y must be float32 or uint16 (bf16 bits)")
    if pos_final.max(initial=-1) >= y.shape[0]:
        raise ValueError("oracle combine: position outside y")
    if out is None:
        out = np.empty((T, H), y.dtype)
    assert out.flags.c_contiguous and out.dtype == y.dtype and out.shape == (T, H)
    rc = _load().monta_oracle_combine(ctypes.c_int64(T), H, k, dtype, _p(y), _p(gates), _p(pos_final), _p(out))
    _check(rc, "combine")
    return out


def unregather(y: np.ndarray, pl: Plan, tp: int, S: int, y_stage: np.ndarray | None = None, slice_: int = -1,
               fill: int = 0) -> np.ndarray:
    """Expert output y [R,H] in FINAL layout -> the unit-major (STAGE) layout, block by block."""
    y = np.ascontiguousarray(y)
    H = y.shape[1]
    E = pl.counts.shape[0]
    if y_stage is None:
        y_stage = np.full((pl.R, H), fill, dtype=y.dtype)
    rc = _load().monta_oracle_unregather(tp, S, E, ctypes.c_int64(H * y.itemsize), _p(pl.n), _p(pl.stage_off),
                                         _p(pl.unit_base), _p(y), _p(y_stage), slice_)
    _check(rc, "unregather")
    return y_stage


def combine_staged(y_stage: np.ndarray, gates: np.ndarray, pos_stage: np.ndarray, out: np.ndarray | None = None,
                   t0: int = 0, t1: int | None = None) -> np.ndarray:
    """Scale-add from the unit-major layout for tokens [t0, t1)."""
    y_stage = np.ascontiguousarray(y_stage)
    gates = np.ascontiguousarray(gates, dtype=np.float32)
    pos_stage = np.ascontiguousarray(pos_stage, dtype=np.int32)
    T, k = pos_stage.shape
    H = y_stage.shape[1]
    t1 = T if t1 is None else t1
    dtype = 0 if y_stage.dtype == np.float32 else 1
    if y_stage.dtype not in (np.float32, np.uint16):
        raise ValueError("oracle combine_staged: y_stage must be float32 or uint16 (bf16 bits)")
    if pos_stage.max(initial=-1) >= y_stage.shape[0]:
        raise ValueError("oracle combine_staged: position outside y_stage")
    if out is None:
        out = np.zeros((T, H), y_stage.dtype)
    rc = _load().monta_oracle_combine_staged(ctypes.c_int64(t0), ctypes.c_int64(t1), H, k, dtype, _p(y_stage),
                                             _p(gates), _p(pos_stage), _p(out))
    _check(rc, "combine_staged")
    return out


def volume(pl: Plan, tp: int, S: int, row_bytes: int):
    """-> (unit_bytes [U], dest_bytes [U,ep], slice_gather_bytes [S]) as int64."""
    U, E = pl.n.shape
    ep = pl.send_rows.shape[1]
    unit_bytes = np.empty(U, np.int64)
    dest_bytes = np.empty((U, ep), np.int64)
    slice_bytes = np.empty(S, np.int64)
    rc = _load().monta_oracle_volume(tp, S, E, ep, ctypes.c_int64(row_bytes), _p(pl.n), _p(pl.send_rows),
                                     _p(unit_bytes), _p(dest_bytes), _p(slice_bytes))
    _check(rc, "volume")
    return unit_bytes, dest_bytes, slice_bytes


def expert_ranges(pl: "Plan", tp: int, S: int, slice: int = -1):
    """Row ranges [lo, hi) of every expert in the expert-major buffer: the whole kept segment, or the part
    of it that the tokens of one slice fill (token order inside a segment makes that one contiguous run)."""
    E = pl.kept.shape[0]
    lo = np.asarray(pl.offsets[:E], np.int32).copy()
    hi = (lo + np.asarray(pl.kept, np.int32)).astype(np.int32)
    if slice >= 0:
        ub = np.asarray(pl.unit_base, np.int32).reshape(S * tp, E)
        lo = ub[slice * tp].copy()
        if slice + 1 < S:
            hi = ub[(slice + 1) * tp].copy()
    return np.ascontiguousarray(lo), np.ascontiguousarray(hi)


def expert(x_final: np.ndarray, w: np.ndarray, seg_lo: np.ndarray, seg_hi: np.ndarray, y: np.ndarray | None = None,
           only_rows=None) -> np.ndarray:
    """One linear layer per expert on the expert-major buffer: y[r] = x_final[r] @ w[e].T for rows r of expert e's
    range.  x_final [rows, H], w [E, N, H], same dtype (float32 or uint16 bf16 bits); y [rows, N] is created
    zero-filled if not given; rows outside every range stay as they are."""
    x_final = np.ascontiguousarray(x_final)
    w = np.ascontiguousarray(w)
    if x_final.dtype != w.dtype or x_final.dtype not in (np.float32, np.uint16) or w.ndim != 3 or w.shape[2] != x_final.shape[1]:
        raise ValueError("oracle expert: x_final [rows,H] and w [E,N,H] must share dtype (float32 or uint16) and H")
    E, N, H = w.shape
    if y is None:
        y = np.zeros((x_final.shape[0], N), x_final.dtype)
    assert y.flags.c_contiguous and y.dtype == x_final.dtype and y.shape == (x_final.shape[0], N)
    lo = np.ascontiguousarray(seg_lo, np.int32)
    hi = np.ascontiguousarray(seg_hi, np.int32)
    assert lo.shape == (E,) and hi.shape == (E,) and int(hi.max(initial=0)) <= x_final.shape[0]
    rows = None if only_rows is None else np.ascontiguousarray(only_rows, np.int32)
    rc = _load().monta_oracle_expert(E, H, N, 0 if x_final.dtype == np.float32 else 1, _p(lo), _p(hi), _p(x_final), _p(w),
                                     _p(y), None if rows is None else _p(rows), ctypes.c_int64(0 if rows is None else rows.size))
    _check(rc, "expert")
    return y


@dataclass
class Result:
    topk_idx: np.ndarray
    gates: np.ndarray
    plan: Plan
    stage: np.ndarray
    final: np.ndarray
    out: np.ndarray


def forward(logits, x, *, k, ep, tp, S, cf, renorm=1, padded=0, fill=0, reuse: Result | None = None) -> Result:
    """The whole path with identity experts (expert output = FINAL).  `reuse`: a result of the same problem whose
    STAGE / FINAL / out arrays are written again instead of allocating fresh ones (for timing without page faults)."""
    E = logits.shape[1]
    idx, gates = route(logits, k, renorm)
    pl = plan(idx, E, ep, tp, S, cf, padded)
    stage = pack(x, pl, tp, S, stage=None if reuse is None else reuse.stage)
    final = regather(stage, pl, tp, S, final=None if reuse is None else reuse.final, fill=fill)
    if padded:
        pad(final, pl)
    out = combine(final, gates, pl.pos_final, out=None if reuse is None else reuse.out)
    return Result(idx, gates, pl, stage, final, out)
