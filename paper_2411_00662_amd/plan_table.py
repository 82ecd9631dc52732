"""The paper's strategy choice (Algorithms 1-3 of section "Network-traffic-aware") run with the D2D-copy
efficiency curve r3 that `r3_sweep` measured on this GPU, for the sequence lengths of Table 7.

Inputs.  Traffic I = b*s*h*BPE (Eq. 3) with h = 8192 and b*BPE = 4, the reading under which s = 8K gives
Table 8's 256 M; t = 8, e = 2 (Table 7).  The two network legs keep the paper's own figures, because this
build has no network: B1 = 25 GB/s, B2 = 200 GB/s and the efficiency samples of Table 8 (r1: 8 M 42.7 %,
32 M 63.2 %, 256 M 74.1 %; r2: 64 M 72.6 %, 256 M 77.6 %).  Only the memory leg is this machine's:
B3 = 8 TB/s (HBM3E peak) and r3(volume) from profiles/r3_regather_mi355x.txt (payload over time over B3).

  python -m paper_2411_00662_amd.plan_table [r3 file]

prints one line per sequence length: the three strategy costs, the chunk counts and the chosen strategy.
"""
from __future__ import annotations

import os
import sys

from . import binding as B

M = 1e6
R1 = [(8 * M, 0.427), (32 * M, 0.632), (256 * M, 0.741)]
R2 = [(64 * M, 0.726), (256 * M, 0.776)]
SEQ_LENGTHS = [4096, 8192, 16384, 32768, 65536, 131072, 262144]       # Table 7: 4K ... 256K
DEFAULT_R3 = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "r3_regather_mi355x.txt")


def read_r3(path: str = DEFAULT_R3):
    """(payload bytes, r3) samples from the summary r3_sweep writes."""
    pts = []
    for line in open(path):
        if line.startswith("#") or not line.strip() or line.lstrip().startswith("payload"):
            continue
        f = line.split()
        pts.append((float(f[0]) * 2 ** 20, float(f[2])))
    if not pts:
        raise ValueError(f"no r3 samples in {path}")
    return sorted(pts)


def traffic_of(seq_len: int) -> float:
    return 4.0 * seq_len * 8192            # b*BPE = 4, h = 8192


def plan_table(r3, seq_lengths=SEQ_LENGTHS, b3=8e12, i_minimal=1e6, n_max=64):
    rows = []
    for s in seq_lengths:
        pin, keep = B.make_plan_in(traffic_of(s), 8, 2, 25e9, 200e9, b3, R1, R2, r3, i_minimal, n_max)
        out = B.monta_plan_strategy(pin)
        rows.append({"seq": s, "traffic": traffic_of(s), "t_base": out.t_base, "t_o1": out.t_o1, "t_o2": out.t_o2,
                     "n_o2": out.n_o2, "t_o3": out.t_o3, "n_o3": out.n_o3, "strategy": out.strategy, "chunks": out.chunks})
    return rows


def main(path=DEFAULT_R3):
    r3 = read_r3(path)
    print(f"# r3 from {os.path.basename(path)}: {len(r3)} samples, {r3[0][1]:.3f} at {r3[0][0] / 2**20:.0f} MiB ... "
          f"{r3[-1][1]:.3f} at {r3[-1][0] / 2**20:.0f} MiB; B3 = 8 TB/s")
    print(f"{'seq':>7s} {'I_MB':>8s} {'base_ms':>9s} {'O1_ms':>8s} {'O2_ms':>8s} {'N_O2':>5s} {'O3_ms':>8s} {'N_O3':>5s} {'chosen':>7s} {'vs_base':>8s}")
    for r in plan_table(r3):
        best = min(r["t_o1"], r["t_o2"], r["t_o3"])
        print(f"{r['seq']:7d} {r['traffic'] / 1e6:8.0f} {r['t_base'] * 1e3:9.3f} {r['t_o1'] * 1e3:8.3f} {r['t_o2'] * 1e3:8.3f} "
              f"{r['n_o2']:5d} {r['t_o3'] * 1e3:8.3f} {r['n_o3']:5d} {'O%d' % r['strategy']:>7s} {best / r['t_base']:8.3f}")


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else DEFAULT_R3)
