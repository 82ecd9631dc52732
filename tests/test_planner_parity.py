"""The library's planner (monta_plan_*, host code in libmonta.so) against the Python reference.
Both are fp64 evaluations of the same closed forms, so results must agree to rounding order."""
import math
import random

import pytest

import paper_2411_00662_amd as m
from oracle import planner as P

M = 1e6
R1 = [(8 * M, 0.427), (32 * M, 0.632), (256 * M, 0.741)]
R2 = [(64 * M, 0.726), (256 * M, 0.776)]
R3 = [(64 * M, 0.80)]


def both(I, t, e, B1, r1, B2, r2, B3, r3, imin, n_max=1 << 16):
    pin, keep = m.make_plan_in(I, t, e, B1, B2, B3, r1, r2, r3, imin, n_max)
    out = m.monta_plan_strategy(pin)
    name, costs = P.select(I, t, e, B1, r1, B2, r2, B3, r3, imin, n_max)
    return pin, out, name, costs


def test_table8_workload():
    pin, out, name, costs = both(256 * M, 8, 2, 25e9, R1, 200e9, R2, 1.6e12, R3, 1e6)
    assert out.t_base == pytest.approx(P.t_base(256 * M, 2, 25e9, R1), rel=1e-12)
    assert math.floor(out.t_base * 1e6) / 1e3 == 6.909            # Table 8, baseline row
    assert out.t_o1 == pytest.approx(costs["O1"][1], rel=1e-12)
    assert (out.n_o2, out.n_o3) == (costs["O2"][0], costs["O3"][0])
    assert out.t_o2 == pytest.approx(costs["O2"][1], rel=1e-12) and out.t_o3 == pytest.approx(costs["O3"][1], rel=1e-12)
    assert out.strategy == {"O1": 1, "O2": 2, "O3": 3}[name]
    aa, ag, d2d = m.monta_plan_chunk_times(pin, 4)
    ref = P.chunk_times(256 * M, 4, 8, 2, 25e9, R1, 200e9, R2, 1.6e12, R3)
    assert (aa, ag, d2d) == pytest.approx(ref, rel=1e-12)
    assert [math.floor(v * 1e6) / 1e3 for v in (aa, ag)] == [0.374, 0.385] and d2d * 1e3 == pytest.approx(0.05)


def test_random_problems_agree():
    rng = random.Random(5)
    for _ in range(300):
        I = 10 ** rng.uniform(5, 10.5)
        t, e = rng.choice([1, 2, 4, 8, 16]), rng.choice([1, 2, 4, 8, 64])
        B1, B2, B3 = 10 ** rng.uniform(9.5, 11), 10 ** rng.uniform(10.5, 12), 10 ** rng.uniform(12, 13)

        def curve():
            n = rng.randint(1, 6)
            xs = sorted(10 ** rng.uniform(4, 10) for _ in range(n))
            xs = [x * (1 + 1e-3 * i) for i, x in enumerate(xs)]
            return [(x, rng.uniform(0.05, 1.0)) for x in xs]

        r1, r2, r3 = curve(), curve(), curve()
        imin = 10 ** rng.uniform(3, 7)
        n_max = rng.choice([1, 7, 64, 1 << 12])
        pin, out, name, costs = both(I, t, e, B1, r1, B2, r2, B3, r3, imin, n_max)
        assert out.t_o1 == pytest.approx(costs["O1"][1], rel=1e-11)
        for key, n_got, t_got in (("O2", out.n_o2, out.t_o2), ("O3", out.n_o3, out.t_o3)):
            n_ref, t_ref = costs[key]
            if n_ref == 0:
                assert n_got == 0 and math.isinf(t_got)
            else:
                assert t_got == pytest.approx(t_ref, rel=1e-11)
                if n_got != n_ref:       # two chunk counts within rounding of each other
                    alt = P.t_chunked(I, n_got, t, e, B1, r1, B2, r2, B3, r3, key == "O3")
                    assert alt == pytest.approx(t_ref, rel=1e-11)
        best = min(costs[k][1] for k in costs)
        assert out.t_best == pytest.approx(best, rel=1e-11)
        assert {1: "O1", 2: "O2", 3: "O3"}[out.strategy] == name or costs[{1: "O1", 2: "O2", 3: "O3"}[out.strategy]][1] == pytest.approx(best, rel=1e-11)


def test_bad_inputs_are_rejected():
    pin, keep = m.make_plan_in(256 * M, 8, 2, 25e9, 200e9, 1.6e12, R1, R2, R3, 1e6)
    for field, value in [("traffic", 0.0), ("traffic", float("nan")), ("t", 0), ("e", 0), ("b1", 0.0), ("b3", -1.0),
                         ("i_minimal", -1.0), ("n_max", 0)]:
        old = getattr(pin, field)
        setattr(pin, field, value)
        with pytest.raises(m.MontaError):
            m.monta_plan_strategy(pin)
        setattr(pin, field, old)
    bad, keep2 = m.make_plan_in(256 * M, 8, 2, 25e9, 200e9, 1.6e12, [(2.0, 0.5), (1.0, 0.6)], R2, R3, 1e6)   # not ascending
    with pytest.raises(m.MontaError):
        m.monta_plan_strategy(bad)
    bad, keep3 = m.make_plan_in(256 * M, 8, 2, 25e9, 200e9, 1.6e12, R1, [(1.0, 0.0)], R3, 1e6)               # zero efficiency
    with pytest.raises(m.MontaError):
        m.monta_plan_strategy(bad)
    with pytest.raises(m.MontaError):
        m.monta_plan_chunk_times(pin, 0)


def test_strategy_table_with_the_r3_curve_measured_on_mi355x():
    """Algorithms 1-3 over Table 7's sequence lengths with this GPU's measured D2D-copy efficiency (the file
    under profiles/ that r3_sweep wrote): the library against the Python reference, row by row."""
    from paper_2411_00662_amd import plan_table as pt
    r3 = pt.read_r3()
    assert len(r3) >= 8 and all(0.0 < e <= 1.0 for _, e in r3) and r3 == sorted(r3)
    rows = pt.plan_table(r3)
    assert [r["seq"] for r in rows] == pt.SEQ_LENGTHS
    for r in rows:
        I = pt.traffic_of(r["seq"])
        name, costs = P.select(I, 8, 2, 25e9, pt.R1, 200e9, pt.R2, 8e12, r3, 1e6, 64)
        assert r["t_o1"] == pytest.approx(costs["O1"][1], rel=1e-12)
        assert r["t_o2"] == pytest.approx(costs["O2"][1], rel=1e-12)
        assert r["t_o3"] == pytest.approx(costs["O3"][1], rel=1e-12)
        assert r["strategy"] == {"O1": 1, "O2": 2, "O3": 3}[name]
        assert r["t_base"] == pytest.approx(P.t_base(I, 2, 25e9, pt.R1), rel=1e-12)
        # every transform beats the plain AllToAll, and pipelining the copy too (O3) is never worse than O2
        assert r["t_o3"] <= r["t_o2"] < r["t_o1"] < r["t_base"]
    # at 8K the traffic is Table 8's 256 M (2^28 bytes under b*BPE = 4)
    assert pt.traffic_of(8192) == 2 ** 28
    # with the memory leg of this GPU the D2D copy of a 64 MiB chunk costs a twentieth of its gather
    pin, keep = m.make_plan_in(pt.traffic_of(8192), 8, 2, 25e9, 200e9, 8e12, pt.R1, pt.R2, r3, 1e6, 64)
    aa, ag, d2d = m.monta_plan_chunk_times(pin, 4)
    assert d2d < ag / 10 and d2d == pytest.approx(2 ** 26 / (8e12 * P.lookup(r3, 2 ** 26)), rel=1e-12)
