"""Device-buffer plumbing on top of the binding: allocation with torch and reading
the plan tables back from the workspace.  No step of the method runs here."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import binding as B


@dataclass
class Buffers:
    cfg: B.monta_cfg
    layout: B.monta_ws_layout
    logits: "torch.Tensor"
    x: "torch.Tensor"
    topk_idx: "torch.Tensor"
    gates: "torch.Tensor"
    ws: "torch.Tensor"
    stage: "torch.Tensor"
    final: "torch.Tensor"
    out: "torch.Tensor"


def _act_dtype(cfg):
    import torch
    return torch.float32 if cfg.dtype == B.FP32 else torch.bfloat16


def to_device_act(cfg, x_host: np.ndarray):
    """Host activations (float32, or uint16 bf16 bit patterns) -> device tensor of cfg's dtype."""
    import torch
    if cfg.dtype == B.FP32:
        return torch.from_numpy(np.ascontiguousarray(x_host, dtype=np.float32)).cuda()
    bits = np.ascontiguousarray(x_host, dtype=np.uint16)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_host_act(cfg, t, rows=None) -> np.ndarray:
    """Device activations -> numpy (float32, or uint16 bf16 bit patterns)."""
    import torch
    if rows is not None:
        t = t[:rows]
    if cfg.dtype == B.FP32:
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def alloc_buffers(cfg, logits_host=None, x_host=None, canary: int | None = None, device="cuda:0") -> Buffers:
    """Allocates every buffer of the path at its worst-case size and initialises the workspace.

    canary: if given, STAGE / FINAL / out are filled with this byte so that tests can see
    which rows were written."""
    import torch
    L = B.monta_ws_layout_query(cfg)
    T, H, E, k = cfg.tokens, cfg.hidden, cfg.experts, cfg.top_k
    dt = _act_dtype(cfg)
    with torch.cuda.device(device):
        logits = (torch.from_numpy(np.ascontiguousarray(logits_host, dtype=np.float32)).cuda()
                  if logits_host is not None else torch.empty((T, E), dtype=torch.float32, device=device))
        x = to_device_act(cfg, x_host) if x_host is not None else torch.empty((T, H), dtype=dt, device=device)
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=device)
        gates = torch.empty((T, k), dtype=torch.float32, device=device)
        ws = torch.zeros(L.ws_bytes, dtype=torch.uint8, device=device)
        stage = torch.empty((L.max_rows, H), dtype=dt, device=device)
        final = torch.empty((L.max_rows, H), dtype=dt, device=device)
        out = torch.empty((T, H), dtype=dt, device=device)
        if canary is not None:
            for t in (stage, final, out):
                t.view(torch.uint8).fill_(canary)
        B.monta_ws_init(cfg, ws)
    return Buffers(cfg, L, logits, x, topk_idx, gates, ws, stage, final, out)


_TABLES = [("meta", "off_meta", lambda c, L: (16,)),
           ("counts", "off_counts", lambda c, L: (c.experts,)),
           ("kept", "off_kept", lambda c, L: (c.experts,)),
           ("offsets", "off_offsets", lambda c, L: (c.experts + 1,)),
           ("n", "off_n", lambda c, L: (L.units, c.experts)),
           ("stage_off", "off_stage_off", lambda c, L: (L.units, c.experts)),
           ("unit_base", "off_unit_base", lambda c, L: (L.units, c.experts)),
           ("send_rows", "off_send_rows", lambda c, L: (L.units, c.ep)),
           ("unit_rows", "off_unit_rows", lambda c, L: (L.units + 1,)),
           ("pos_final", "off_pos_final", lambda c, L: (c.tokens, c.top_k)),
           ("pos_stage", "off_pos_stage", lambda c, L: (c.tokens, c.top_k)),
           ("row_map", "off_row_map", lambda c, L: (L.max_rows,))]


def read_tables(cfg, ws) -> dict:
    """Copies the plan tables out of a device workspace into numpy int32 arrays."""
    L = B.monta_ws_layout_query(cfg)
    host = ws.cpu().numpy()
    out = {}
    for name, off_name, shape_fn in _TABLES:
        shape = shape_fn(cfg, L)
        cnt = int(np.prod(shape))
        off = getattr(L, off_name)
        out[name] = host[off:off + 4 * cnt].view(np.int32).reshape(shape).copy()
    out["kept_prefix"] = host[L.off_kept_prefix:L.off_kept_prefix + 4 * (cfg.experts + 1)].view(np.int32).copy()
    out["final_rows"] = int(out["meta"][4])
    out["R"] = int(out["meta"][0])
    out["alive"] = int(out["meta"][1])
    out["C"] = int(out["meta"][2])
    return out
