"""Fused regather against the paper's two-pass orders (gather, then D2D copy), per chunk payload, on this GPU.

For every payload the same problem (hidden 8192 bf16, 2 experts, top-1, tp 8, 4 chunks: the paper's evaluation
shape) is packed once, then four ways of getting STAGE into FINAL are timed back to back, each replayed from a
captured HIP graph:

  fused      monta_regather, slice by slice (gather + copy in one pass)
  serial     monta_allgather_regather(schedule 0): gather(j), copy(j), one stream, nothing overlaps (O2 order)
  cosched    monta_allgather_regather(schedule 1): copy(j) and gather(j+1) in one grid (O3 order)
  streams    monta_allgather_regather(schedule 2): gathers and copies on two streams with events (O3 order,
             the paper's stream picture)

The question the paper raises in its discussion is whether the overlapped kernels interfere at small volumes.

  python -m paper_2411_00662_amd.twopass_sweep [out.txt]
"""
from __future__ import annotations

import sys


def main(out_path=None):
    import numpy as np
    import torch
    import paper_2411_00662_amd as m

    H, E, k, ep, tp, S = 8192, 2, 1, 2, 8, 4
    lines = ["# regather of 4 chunks, hidden 8192 bf16 (16 KiB rows), 2 experts, top-1, tp 8: time for all 4 chunks, us",
             "# payload = bytes one chunk's gather (or copy) reads; fused moves 2 x payload per chunk, the two-pass orders 4 x",
             f"{'payload_MiB':>11s} {'fused':>9s} {'serial':>9s} {'cosched':>9s} {'streams':>9s} {'cosched/serial':>15s} {'streams/serial':>15s}"]
    stream = torch.cuda.Stream()
    for mib in (1, 2, 4, 8, 16, 32, 64, 128):
        T = (mib << 20) // (H * 2) * S           # tokens so that one chunk carries `mib` MiB
        cfg = m.make_cfg(T, H, m.BF16, E, k, ep, tp, S, 0.0)
        rng = np.random.default_rng(mib)
        logits = rng.standard_normal((T, E), dtype=np.float32)
        b = m.alloc_buffers(cfg, logits, None)
        b.x.view(torch.int16).random_(-2000, 2000)
        gathered = torch.empty_like(b.stage)
        with torch.cuda.stream(stream):
            m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws, stream)
            m.monta_dispatch(cfg, b.x, b.stage, b.ws, -1, stream)

            def fused():
                for j in range(S):
                    m.monta_regather(cfg, b.stage, b.final, b.ws, j, stream)

            def two_pass(schedule):
                return lambda: m.monta_allgather_regather(cfg, b.stage, gathered, b.final, b.ws, schedule, stream)

            res = []
            for fn in (fused, two_pass(0), two_pass(1), two_pass(2)):
                for _ in range(3):
                    fn()
                stream.synchronize()
                # replayed from a captured graph, so that what is timed is the GPU's work and its launch
                # boundaries, not the host's calls (the variants differ in how many calls they are)
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    fn()
                for _ in range(5):
                    graph.replay()
                torch.cuda.synchronize()
                reps = 50 if mib <= 16 else 20
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                res.append(e0.elapsed_time(e1) * 1e3 / reps)
                del graph
        lines.append(f"{mib:11d} {res[0]:9.1f} {res[1]:9.1f} {res[2]:9.1f} {res[3]:9.1f} {res[2] / res[1]:15.3f} {res[3] / res[1]:15.3f}")
        print(lines[-1], flush=True)
        del b, gathered
    if out_path:
        with open(out_path, "w") as f:
            f.write("# command: python -m paper_2411_00662_amd.twopass_sweep\n" + "\n".join(lines) + "\n")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else None)
