"""Measures r3, the memory-bandwidth utilisation of the D2D copy stage (Eq. 10 of the paper), on this GPU:
the regather kernel's payload rate against the HBM peak, as a function of the chunk payload I/N.

  python -m paper_2411_00662_amd.r3_sweep [out.txt]

Eq. 10 counts the payload once (a copy reads and writes it), so r3 = payload / (time * B3) with
B3 = 8 TB/s; the read+write rate is twice the payload rate.  The table can be fed to
monta_plan_strategy as the r3 curve.
"""
from __future__ import annotations

import sys

import numpy as np

B3 = 8.0e12


def main(out_path=None):
    import torch
    import paper_2411_00662_amd as m

    lines = ["# regather (gather + D2D copy stage) on one MI355X: hidden 8192 bf16 rows, 2 experts, top-1, one slice",
             "# r3 = payload / (time * 8 TB/s); the kernel reads and writes the payload once each;",
             "# time = average over back-to-back launches, launch latency included (the fixed overhead of a chunk)",
             f"{'payload_MiB':>12s} {'time_us':>10s} {'r3':>8s} {'read+write_GBps':>16s}"]
    H, E = 8192, 2
    for mib in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024):
        T = mib * (1 << 20) // (H * 2)
        cfg = m.make_cfg(T, H, m.BF16, E, 1, 2, 1, 1, 0.0)
        rng = np.random.default_rng(0)
        logits = rng.standard_normal((T, E), dtype=np.float32)
        b = m.alloc_buffers(cfg, logits, None)
        b.x.zero_()
        m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
        m.monta_dispatch(cfg, b.x, b.stage, b.ws, -1)
        reps = 200 if mib <= 64 else 30
        # raw C calls with the pointers marshalled once: the loop must stay GPU-bound for small payloads
        import ctypes
        fn = m.binding.lib().monta_regather
        args = (ctypes.byref(cfg), b.stage.data_ptr(), b.final.data_ptr(), b.ws.data_ptr(), 0,
                torch.cuda.current_stream().cuda_stream)
        for _ in range(5):
            assert fn(*args) == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn(*args)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        payload = T * H * 2
        lines.append(f"{mib:12d} {us:10.2f} {payload / (us * 1e-6) / B3:8.4f} {2 * payload / (us * 1e-6) / 1e9:16.1f}")
        print(lines[-1], flush=True)
        del b
    if out_path:
        with open(out_path, "w") as f:
            f.write("# command: python -m paper_2411_00662_amd.r3_sweep\n" + "\n".join(lines) + "\n")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else None)
