"""Pins of the planner reference (oracle/planner.py) to the numbers the paper prints."""
import math
import os

import pytest

from oracle import planner as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table8_model.txt")
M = 1e6


def golden():
    rows, scal = {}, {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 4:
            rows[line[0]] = tuple(float(v) for v in line[1:])
        elif len(line) == 2:
            scal[line[0]] = float(line[1])
    return rows, scal


ROWS, SCAL = golden()
B1, B2 = SCAL["B1_GBps"] * 1e9, SCAL["B2_GBps"] * 1e9
T_, E_ = 8, 2
I = ROWS["baseline_alltoall"][0] * M
# D2D row: 64 M at 80 % in 0.05 ms  =>  B3 = 64e6 / (0.05e-3 * 0.8)
B3 = ROWS["chunk4_d2d"][0] * M / (ROWS["chunk4_d2d"][2] * 1e-3 * ROWS["chunk4_d2d"][1])
R1 = [(ROWS["chunk4_alltoall"][0] * M, ROWS["chunk4_alltoall"][1]), (ROWS["o1_alltoall"][0] * M, ROWS["o1_alltoall"][1]),
      (ROWS["baseline_alltoall"][0] * M, ROWS["baseline_alltoall"][1])]
R2 = [(ROWS["chunk4_allgather"][0] * M, ROWS["chunk4_allgather"][1]), (ROWS["o1_allgather"][0] * M, ROWS["o1_allgather"][1])]
R3 = [(ROWS["chunk4_d2d"][0] * M, ROWS["chunk4_d2d"][1])]


def trunc3(ms):
    return math.floor(ms * 1000 + 1e-9) / 1000


def test_traffic_and_volumes():
    assert P.traffic(1, 8192, 8192, 4) == 2 ** 28          # Eq. 3; Table 8 rounds this to 256 M
    assert I / T_ == ROWS["o1_alltoall"][0] * M            # 1/t of the volume after the split
    assert I / (4 * T_) == ROWS["chunk4_alltoall"][0] * M
    assert I / 4 == ROWS["chunk4_allgather"][0] * M == ROWS["chunk4_d2d"][0] * M
    assert B3 == pytest.approx(1.6e12)


def test_table8_latencies_from_eq_8_to_11():
    assert trunc3(P.t_base(I, E_, B1, R1) * 1e3) == ROWS["baseline_alltoall"][2]
    aa, ag, d2d = P.chunk_times(I, 4, T_, E_, B1, R1, B2, R2, B3, R3)
    assert trunc3(aa * 1e3) == ROWS["chunk4_alltoall"][2]
    assert trunc3(ag * 1e3) == ROWS["chunk4_allgather"][2]
    assert d2d * 1e3 == pytest.approx(ROWS["chunk4_d2d"][2])
    # Eq. 11 is the sum of the two O1 rows
    o1_aa = I / T_ * (E_ - 1) / E_ / (B1 * ROWS["o1_alltoall"][1])
    o1_ag = I * (T_ - 1) / T_ / (B2 * ROWS["o1_allgather"][1])
    assert trunc3(o1_aa * 1e3) == ROWS["o1_alltoall"][2] and trunc3(o1_ag * 1e3) == ROWS["o1_allgather"][2]
    assert P.t_o1(I, T_, E_, B1, R1, B2, R2) == pytest.approx(o1_aa + o1_ag, rel=1e-12)
    assert aa / ag == pytest.approx(SCAL["aa_over_ag_printed"], abs=0.01)


def test_printed_ratios():
    # the printed O2 / O3 ratios use a baseline evaluated at the chunked AllToAll efficiency (0.427)
    base_427 = I * (E_ - 1) / E_ / (B1 * ROWS["chunk4_alltoall"][1])
    o2 = P.t_chunked(I, 4, T_, E_, B1, R1, B2, R2, B3, R3, o3=False)
    o3 = P.t_chunked(I, 4, T_, E_, B1, R1, B2, R2, B3, R3, o3=True)
    assert o2 / base_427 == pytest.approx(SCAL["ratio_o2_printed"], abs=1e-3)
    assert o3 / base_427 == pytest.approx(SCAL["ratio_o3_printed"], abs=1e-3)
    assert o3 < o2                                       # pipelining the D2D copy can only help in the model
    # the printed O1 ratio 0.31 uses the baseline at the O1 AllToAll efficiency (0.632)
    base_632 = I * (E_ - 1) / E_ / (B1 * ROWS["o1_alltoall"][1])
    assert P.t_o1(I, T_, E_, B1, R1, B2, R2) / base_632 == pytest.approx(SCAL["ratio_o1_printed"], abs=0.01)


def test_eq12_and_eq13_closed_forms():
    flat = [(1.0, 0.75)]                                 # r1 = r2 at every volume
    r3_free = [(1.0, 1.0)]
    aa, ag, _ = P.chunk_times(I, 4, T_, E_, B1, flat, B2, flat, 1e30, r3_free)
    assert aa / ag == pytest.approx(SCAL["eq12_ratio"], rel=1e-9)           # (e-1) B2 / (e (t-1) B1) = 4/7
    base = P.t_base(I, E_, B1, flat)
    ratios = [P.t_chunked(I, n, T_, E_, B1, flat, B2, flat, 1e30, r3_free, o3=True) / base for n in (4, 64, 4096)]
    assert ratios[0] > ratios[1] > ratios[2] > SCAL["eq13_limit"]
    assert ratios[2] == pytest.approx(SCAL["eq13_limit"], rel=1e-3)         # -> 7/32 as N grows
    assert SCAL["measured_o3_256k"] > SCAL["eq13_limit"]                    # the measured 0.253 sits above the bound


def test_search_and_selection():
    # no fixed overhead in the curves => more chunks always help until chunks hit I_minimal
    flat = [(1.0, 0.75)]
    n2, t2 = P.search(I, T_, E_, B1, flat, B2, flat, B3, [(1.0, 0.8)], i_minimal=1e6, o3=False)
    assert n2 == 32                                      # I/(N t) >= 1e6  <=>  N <= 32
    for n in range(1, 33):
        assert t2 <= P.t_chunked(I, n, T_, E_, B1, flat, B2, flat, B3, [(1.0, 0.8)], o3=False) + 1e-18
    assert P.search(1e5, T_, E_, B1, flat, B2, flat, B3, flat, i_minimal=1e6, o3=True) == (0, math.inf)
    # with the paper's efficiency points small chunks are inefficient: the search must not run to the limit
    name, costs = P.select(I, T_, E_, B1, R1, B2, R2, B3, R3, i_minimal=1e6)
    assert set(costs) == {"O1", "O2", "O3"} and name == min(costs, key=lambda k: costs[k][1])
    assert costs["O3"][1] <= costs["O2"][1]
    # tiny traffic: chunking impossible, O1 is selected
    name, costs = P.select(4e6, T_, E_, B1, R1, B2, R2, B3, R3, i_minimal=1e6)
    assert name == "O1" and costs["O2"][0] == 0


def test_lookup_interpolates_and_clamps():
    c = [(10.0, 0.2), (20.0, 0.4), (40.0, 0.8)]
    assert P.lookup(c, 5) == 0.2 and P.lookup(c, 100) == 0.8
    assert P.lookup(c, 15) == pytest.approx(0.3) and P.lookup(c, 30) == pytest.approx(0.6)
    assert P.lookup(c, 20) == pytest.approx(0.4)


def test_lookup_volumes_and_the_alltoall_bound_branch():
    # efficiency curves that differ at every volume involved, so a lookup at the wrong volume shows
    I, t, e, N = 64e6, 4, 2, 2
    b1, b2, b3 = 10e9, 100e9, 1e12
    r1 = [(1e6, 0.1), (1e9, 0.9)]
    r2 = [(1e6, 0.2), (1e9, 0.8)]
    r3 = [(1e6, 0.3), (1e9, 0.7)]

    def lin(c, v):
        (x0, y0), (x1, y1) = c
        return y0 + (y1 - y0) * (v - x0) / (x1 - x0)

    aa, ag, d2d = P.chunk_times(I, N, t, e, b1, r1, b2, r2, b3, r3)
    assert aa == pytest.approx(I / (N * t) * 0.5 / (b1 * lin(r1, I / (N * t))), rel=1e-12)    # r1 at I/(N t)
    assert ag == pytest.approx(I / N * 0.75 / (b2 * lin(r2, I / N)), rel=1e-12)                # r2 at I/N
    assert d2d == pytest.approx(I / N / (b3 * lin(r3, I / N)), rel=1e-12)                      # r3 at I/N
    assert P.t_o1(I, t, e, b1, r1, b2, r2) == pytest.approx(
        I / t * 0.5 / (b1 * lin(r1, I / t)) + I * 0.75 / (b2 * lin(r2, I)), rel=1e-12)       # r1 at I/t, r2 at I
    # slow AllToAll: the chunked pipelines are bound by it, the gather (and copy) of the last chunk trail behind
    slow = 0.2e9
    aa, ag, d2d = P.chunk_times(I, 4, t, e, slow, r1, b2, r2, b3, r3)
    assert aa > ag + d2d
    assert P.t_chunked(I, 4, t, e, slow, r1, b2, r2, b3, r3, o3=False) == pytest.approx(aa * 4 + ag + d2d, rel=1e-12)
    assert P.t_chunked(I, 4, t, e, slow, r1, b2, r2, b3, r3, o3=True) == pytest.approx(aa * 4 + ag + d2d, rel=1e-12)
    # fast AllToAll: the gather stage bounds; Algorithm 1 pays the copy per chunk, Algorithm 2 once
    fast = 1e12
    aa, ag, d2d = P.chunk_times(I, 4, t, e, fast, r1, b2, r2, b3, r3)
    assert aa < ag
    assert P.t_chunked(I, 4, t, e, fast, r1, b2, r2, b3, r3, o3=False) == pytest.approx(aa + 4 * (ag + d2d), rel=1e-12)
    assert P.t_chunked(I, 4, t, e, fast, r1, b2, r2, b3, r3, o3=True) == pytest.approx(aa + 4 * ag + d2d, rel=1e-12)
