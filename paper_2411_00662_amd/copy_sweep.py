"""The achievable copy ceiling of this GPU: the library's plain 16-byte-per-lane copy kernel (monta_copy)
against buffer size, as read+write GB/s and as a fraction of the 8 TB/s HBM peak.

  python -m paper_2411_00662_amd.copy_sweep [out.txt]
"""
from __future__ import annotations

import ctypes
import sys


def main(out_path=None):
    import torch
    import paper_2411_00662_amd as m

    fn = m.binding.lib().monta_copy
    lines = ["# monta_copy (plain copy, 16 bytes per lane, 4 loads in flight, streaming accesses) on one MI355X",
             "# time = average of back-to-back launches on one stream; GB/s counts bytes read + bytes written",
             f"{'buffer_MiB':>11s} {'time_us':>10s} {'GBps':>9s} {'of_8TBps':>9s}"]
    for mib in (16, 32, 64, 128, 256, 512, 1024, 2048, 4096):
        n = mib << 20
        src = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        args = (dst.data_ptr(), src.data_ptr(), ctypes.c_size_t(n), torch.cuda.current_stream().cuda_stream)
        for _ in range(5):
            assert fn(*args) == 0
        torch.cuda.synchronize()
        reps = 100 if mib <= 256 else 20
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn(*args)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        gbps = 2 * n / (us * 1e-6) / 1e9
        lines.append(f"{mib:11d} {us:10.2f} {gbps:9.1f} {gbps / 8000:9.3f}")
        print(lines[-1], flush=True)
        del src, dst
    if out_path:
        with open(out_path, "w") as f:
            f.write("# command: python -m paper_2411_00662_amd.copy_sweep\n" + "\n".join(lines) + "\n")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else None)
