"""Plain Python reference of MoNTA's cost model and strategy search (TEST INFRASTRUCTURE ONLY).

Follows section "Network-traffic-aware": traffic I = b*s*h*BPE (Eq. 3), per-chunk times
AA_j, AG_j, D2D_j (Eq. 8-10), the O1 cost (Eq. 11), the chunk searches (Algorithm 1 for O2,
Algorithm 2 for O3) and the strategy selection (Algorithm 3).  All arithmetic in Python floats
(fp64).  Shares nothing with the product library.

Readings where the printed algorithms are garbled: the loop index j is never used; "T = T_min"
is taken as "remember the best (N, T) seen so far" and the best pair is returned; the search
runs N = 1, 2, ... until a chunk falls under I_minimal (or n_max is reached).  An efficiency
"curve" is a list of (volume in bytes, efficiency) points, interpolated linearly in the volume
and held constant outside the sampled range.
"""
from __future__ import annotations

import math
from bisect import bisect_right


def traffic(b: float, s: float, h: float, bpe: float) -> float:
    """Eq. 3."""
    return b * s * h * bpe


def lookup(curve, volume: float) -> float:
    pts = sorted(curve)
    xs = [p[0] for p in pts]
    if volume <= xs[0]:
        return pts[0][1]
    if volume >= xs[-1]:
        return pts[-1][1]
    i = bisect_right(xs, volume)
    (x0, y0), (x1, y1) = pts[i - 1], pts[i]
    return y0 + (y1 - y0) * (volume - x0) / (x1 - x0)


def t_base(I, e, B1, r1_curve):
    """The untransformed AllToAll: every TP rank sends all of I, the share (e-1)/e leaves the node."""
    return I * (e - 1) / e / (B1 * lookup(r1_curve, I))


def chunk_times(I, N, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve):
    """Eq. 8, 9, 10 for one of N chunks."""
    aa = I / (N * t) * (e - 1) / e / (B1 * lookup(r1_curve, I / (N * t)))
    ag = I / N * (t - 1) / t / (B2 * lookup(r2_curve, I / N))
    d2d = I / N / (B3 * lookup(r3_curve, I / N))
    return aa, ag, d2d


def t_o1(I, t, e, B1, r1_curve, B2, r2_curve):
    """Eq. 11: r1 looked up at I/t, r2 at I."""
    return I / t * (e - 1) / e / (B1 * lookup(r1_curve, I / t)) + I * (t - 1) / t / (B2 * lookup(r2_curve, I))


def t_chunked(I, N, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve, o3: bool):
    aa, ag, d2d = chunk_times(I, N, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve)
    if not o3:      # Algorithm 1: the D2D copy rides in the gather stage
        return aa + (ag + d2d) * N if aa < ag + d2d else aa * N + ag + d2d
    return aa + ag * N + d2d if aa < ag else aa * N + ag + d2d     # Algorithm 2: D2D pipelined too


def search(I, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve, i_minimal, o3: bool, n_max: int = 1 << 16):
    """Algorithms 1 / 2: returns (N, T) of the cheapest chunk count, (0, inf) if even N = 1 is too small."""
    best_n, best_t = 0, math.inf
    n = 1
    while n <= n_max:
        if I / (n * t) < i_minimal or I / n < i_minimal:
            break
        tt = t_chunked(I, n, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve, o3)
        if tt < best_t:
            best_n, best_t = n, tt
        n += 1
    return best_n, best_t


def select(I, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve, i_minimal, n_max: int = 1 << 16):
    """Algorithm 3: the cheapest of O1, O2, O3 (the earlier one wins a tie)."""
    costs = {"O1": (1, t_o1(I, t, e, B1, r1_curve, B2, r2_curve))}
    costs["O2"] = search(I, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve, i_minimal, False, n_max)
    costs["O3"] = search(I, t, e, B1, r1_curve, B2, r2_curve, B3, r3_curve, i_minimal, True, n_max)
    name = min(("O1", "O2", "O3"), key=lambda k: (costs[k][1], ("O1", "O2", "O3").index(k)))
    return name, costs
