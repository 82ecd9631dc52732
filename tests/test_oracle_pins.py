"""CPU-only pins of the oracle.

Every check here compares the oracle with something that is *not* the oracle:
a brute-force definition in Python, a numpy library routine (stable argsort,
bincount, cumsum, dense matrix product), torch's bf16 rounding, a closed form, or
values printed in the paper (tests/golden/).  The checks are chosen so that a
plausible mistake in the oracle (wrong tie-break, dropped term, transposed index,
wrong unit / slice arithmetic, off-by-one in capacity) fails at least one.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads
from workloads import BF16, FP32, Workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers

def brute_topk(logits_row, k):
    """Definition: sort experts by (logit descending, index ascending), take k."""
    E = len(logits_row)
    return sorted(range(E), key=lambda e: (-float(logits_row[e]), e))[:k]


def dense_softmax64(logits):
    z = logits.astype(np.float64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    return p / p.sum(axis=1, keepdims=True)


def ulp32(a):
    return np.spacing(np.abs(a).astype(np.float32)).astype(np.float64)


def brute_plan(idx, E, ep, tp, S, C):
    """Independent formulation: explicit per-expert token lists and sorting by keys."""
    T, k = idx.shape
    U = S * tp
    Tu = T // U
    lists = [[] for _ in range(E)]
    for t in range(T):
        for j in range(k):
            lists[idx[t, j]].append((t, j))
    kept_lists = [l[:C] for l in lists]                      # lowest token indices survive
    final_order = [p for e in range(E) for p in kept_lists[e]]   # expert-major, token order inside
    pos_final = -np.ones((T, k), np.int64)
    for r, (t, j) in enumerate(final_order):
        pos_final[t, j] = r
    # STAGE order: sort the kept pairs by (unit, expert, token)
    stage_order = sorted(final_order, key=lambda p: (p[0] // Tu, idx[p[0], p[1]], p[0]))
    pos_stage = -np.ones((T, k), np.int64)
    for r, (t, j) in enumerate(stage_order):
        pos_stage[t, j] = r
    return lists, kept_lists, final_order, stage_order, pos_final, pos_stage


def rand_case(rng, T, E, k, levels=None):
    if levels:
        return ((rng.integers(0, levels, size=(T, E)).astype(np.float32)) - 1) * np.float32(0.25)
    return rng.standard_normal((T, E), dtype=np.float32)


# ------------------------------------------------------------------ routing

@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (7, 4, 2), (33, 8, 8), (64, 5, 3), (50, 64, 8), (19, 13, 1)])
@pytest.mark.parametrize("ties", [False, True])
def test_route_indices_equal_full_sort(T, E, k, ties):
    rng = np.random.default_rng(100 + T + E + k)
    logits = rand_case(rng, T, E, k, levels=3 if ties else None)
    idx, _ = oracle.route(logits, k)
    for t in range(T):
        assert list(idx[t]) == brute_topk(logits[t], k)
    if ties:
        # with 3 distinct values and E > 3 there must be ties inside some row
        assert any(len(set(logits[t])) < E for t in range(T)) or E == 1


@pytest.mark.parametrize("renorm", [0, 1])
def test_route_gates_equal_dense_softmax(renorm):
    rng = np.random.default_rng(7)
    T, E, k = 200, 16, 4
    logits = rng.standard_normal((T, E), dtype=np.float32) * 3
    idx, gates = oracle.route(logits, k, renorm)
    p = dense_softmax64(logits)
    ref = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        ref = ref / ref.sum(axis=1, keepdims=True)
        np.testing.assert_allclose(gates.astype(np.float64).sum(1), 1.0, atol=2e-7)
    # one rounding to fp32 from an fp64 value that differs from ref by a few fp64 ulps
    assert np.all(np.abs(gates.astype(np.float64) - ref) <= 0.5000001 * ulp32(ref) + 1e-15)
    # gates are sorted like the logits: slot 0 is the strongest
    assert np.all(np.diff(gates, axis=1) <= 0)


def test_route_gates_extreme_logits_do_not_overflow():
    logits = np.array([[80.0, -80.0, 79.0, 0.0], [-90.0, -91.0, -95.0, -200.0]], np.float32)
    idx, gates = oracle.route(logits, 2, 1)
    assert list(idx[0]) == [0, 2] and list(idx[1]) == [0, 1]
    e = math.exp(-1.0)
    np.testing.assert_allclose(gates[0], [1 / (1 + e), e / (1 + e)], rtol=1e-7)
    np.testing.assert_allclose(gates[1], [1 / (1 + e), e / (1 + e)], rtol=1e-7)
    assert np.isfinite(gates).all()
    # far outside the range where exp() of the raw logit is finite in double
    big = np.array([[1000.0, 999.0, -1000.0], [-3000.0, -3001.0, -2999.0]], np.float32)
    idx, gates = oracle.route(big, 2, 0)
    assert list(idx[0]) == [0, 1] and list(idx[1]) == [2, 0]
    np.testing.assert_allclose(gates[0], [1 / (1 + e), e / (1 + e)], rtol=1e-7)
    e2 = math.exp(-2.0)
    np.testing.assert_allclose(gates[1], [1 / (1 + e + e2), e / (1 + e + e2)], rtol=1e-7)


def test_route_k_equals_E_no_renorm_is_plain_softmax():
    rng = np.random.default_rng(3)
    logits = rng.standard_normal((40, 6), dtype=np.float32)
    idx, gates = oracle.route(logits, 6, 0)
    p = dense_softmax64(logits)
    dense = np.zeros_like(p)
    np.put_along_axis(dense, idx.astype(np.int64), gates.astype(np.float64), axis=1)
    np.testing.assert_allclose(dense, p, rtol=1e-7)


def test_route_rejects_nonfinite():
    logits = np.zeros((2, 4), np.float32)
    logits[1, 2] = np.nan
    with pytest.raises(ValueError):
        oracle.route(logits, 2)


# --------------------------------------------------------------------- gate

@pytest.mark.parametrize("dtype", [FP32, BF16])
def test_gate_projection_is_a_matrix_product(dtype):
    w = Workload("t", 50, 96, dtype, 7, 2, 1, 1, 1, 0.0)
    _, x = workloads.make_inputs(w, seed=1)
    wg = workloads.make_gate_weights(w, seed=1)
    got = oracle.gate(x, wg)
    xf = x if dtype == FP32 else workloads.bf16_bits_to_f32(x)
    wf = wg if dtype == FP32 else workloads.bf16_bits_to_f32(wg)
    ref = xf.astype(np.float64) @ wf.astype(np.float64).T            # library routine, its own summation order
    assert got.shape == (50, 7) and got.dtype == np.float32
    assert np.all(np.abs(got.astype(np.float64) - ref) <= 0.5000001 * ulp32(ref) + 1e-12)
    # small integers: every partial sum is exact, so the result must be exact whatever the order
    rng = np.random.default_rng(2)
    xi = rng.integers(-8, 9, size=(20, 64)).astype(np.float32)
    wi = rng.integers(-8, 9, size=(5, 64)).astype(np.float32)
    if dtype == BF16:
        xi_in, wi_in = workloads.f32_to_bf16_bits(xi), workloads.f32_to_bf16_bits(wi)
    else:
        xi_in, wi_in = xi, wi
    np.testing.assert_array_equal(oracle.gate(xi_in, wi_in), (xi.astype(np.int64) @ wi.astype(np.int64).T).astype(np.float32))
    # one-hot weights pick out columns: a transposed operand or a wrong stride would show
    onehot = np.zeros((3, 64), np.float32)
    onehot[0, 5] = onehot[1, 63] = onehot[2, 0] = 1.0
    oh_in = workloads.f32_to_bf16_bits(onehot) if dtype == BF16 else onehot
    np.testing.assert_array_equal(oracle.gate(xi_in, oh_in), xi[:, [5, 63, 0]])


# ------------------------------------------------------------------- expert

def _expert_case(dtype, cf=0.6, seed=4):
    w = Workload("ex", 96, 64, dtype, 6, 2, 3, 2, 2, cf)
    logits, x = workloads.make_inputs(w, seed=seed)
    ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    return w, ref


@pytest.mark.parametrize("dtype", [FP32, BF16])
def test_expert_layer_is_a_matrix_product_per_segment(dtype):
    w, ref = _expert_case(dtype)
    pl = ref.plan
    assert 0 < pl.R < w.tokens * w.top_k and pl.kept.min() > 0
    we = workloads.make_expert_weights(w, n_out=40, seed=1)
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    canary = np.float32(7.0) if dtype == FP32 else np.uint16(0x4123)
    y = np.full((pl.R + 3, 40), canary, dtype=ref.final.dtype)
    xf = np.concatenate([ref.final[:pl.R], np.zeros((3, w.hidden), ref.final.dtype)])
    oracle.expert(xf, we, lo, hi, y)
    as64 = (lambda a: a.astype(np.float64)) if dtype == FP32 else (lambda a: workloads.bf16_bits_to_f32(a).astype(np.float64))
    assert np.all(y[pl.R:] == canary)                               # rows of no expert are not touched
    for e in range(w.experts):
        seg = slice(int(pl.offsets[e]), int(pl.offsets[e] + pl.kept[e]))
        want = as64(xf[seg]) @ as64(we[e]).T                         # library routine, its own summation order
        got = as64(y[seg])
        ulp = ulp32(want) if dtype == FP32 else np.maximum(np.abs(want), 1e-30) * 2.0 ** -7
        assert np.all(np.abs(got - want) <= 0.5000001 * ulp + 1e-12), e
    # power-of-two multiples of the identity: y = 2^e * x exactly, so a row handed to the wrong expert shows
    eye = np.stack([np.eye(w.hidden, dtype=np.float32) * np.float32(2.0 ** e) for e in range(w.experts)])
    eye_in = eye if dtype == FP32 else workloads.f32_to_bf16_bits(eye)
    y2 = oracle.expert(ref.final[:pl.R], eye_in, lo, hi)
    for e in range(w.experts):
        seg = slice(int(pl.offsets[e]), int(pl.offsets[e] + pl.kept[e]))
        np.testing.assert_array_equal(as64(y2[seg]), as64(ref.final[seg]) * 2.0 ** e)


def test_expert_layer_by_slices_and_by_sampled_rows():
    w, ref = _expert_case(BF16)
    pl = ref.plan
    we = workloads.make_expert_weights(w, seed=2)
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    whole = oracle.expert(ref.final[:pl.R], we, lo, hi)
    # the slices' ranges tile every segment in order, and computing slice by slice gives the same buffer
    parts = np.zeros_like(whole)
    covered = np.zeros(pl.R, np.int32)
    prev_hi = lo.copy()
    for j in range(w.slices):
        lj, hj = oracle.expert_ranges(pl, w.tp, w.slices, j)
        np.testing.assert_array_equal(lj, prev_hi)
        prev_hi = hj
        for e in range(w.experts):
            covered[lj[e]:hj[e]] += 1
            # rows of slice j in segment e are exactly the kept pairs of e whose token lies in slice j
            toks = np.nonzero((ref.topk_idx == e).any(axis=1))[0]
            pos = np.array([ref.plan.pos_final[t, list(ref.topk_idx[t]).index(e)] for t in toks])
            in_slice = (toks // (w.tokens // w.slices) == j) & (pos >= 0)
            assert sorted(pos[in_slice]) == list(range(lj[e], hj[e]))
        oracle.expert(ref.final[:pl.R], we, lj, hj, parts)
    np.testing.assert_array_equal(prev_hi, hi)
    assert np.all(covered == 1)
    np.testing.assert_array_equal(parts, whole)
    # a sample of rows: the same values on those rows, nothing else written
    rows = np.array([0, 5, pl.R - 1, int(pl.offsets[3])], np.int32)
    some = oracle.expert(ref.final[:pl.R], we, lo, hi, only_rows=rows)
    np.testing.assert_array_equal(some[rows], whole[rows])
    mask = np.ones(pl.R, bool)
    mask[rows] = False
    assert not some[mask].any()


def test_identity_expert_weights_give_the_identity_expert_path():
    w, ref = _expert_case(BF16, cf=0.0)
    pl = ref.plan
    eye = workloads.f32_to_bf16_bits(np.stack([np.eye(w.hidden, dtype=np.float32)] * w.experts))
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    y = oracle.expert(ref.final[:pl.R], eye, lo, hi)
    np.testing.assert_array_equal(y, ref.final[:pl.R])
    np.testing.assert_array_equal(oracle.combine(y, ref.gates, pl.pos_final), ref.out)


# --------------------------------------------------------------------- plan

def test_capacity_formula():
    # ceil(cf*T*k/E), exact integers for the named workloads, clipped to T, cf=0 => T
    assert oracle.capacity(8192, 8, 2, 2.0) == 4096
    assert oracle.capacity(32768, 8, 2, 1.25) == 10240
    assert oracle.capacity(65536, 64, 8, 1.25) == 10240
    assert oracle.capacity(100, 8, 2, 0.0) == 100
    assert oracle.capacity(10, 3, 2, 1.0) == 7          # ceil(6.67)
    assert oracle.capacity(10, 2, 2, 4.0) == 10         # clipped to T
    assert oracle.capacity(7, 4, 1, 0.5) == 1           # ceil(0.875)


@pytest.mark.parametrize("T,E,k,ep,tp,S,cf", [
    (24, 4, 2, 2, 2, 2, 0.0),
    (24, 4, 2, 2, 2, 3, 0.5),
    (60, 6, 3, 3, 5, 2, 0.75),
    (64, 8, 1, 8, 1, 1, 0.0),
    (64, 8, 8, 1, 4, 4, 0.6),
    (30, 5, 2, 1, 3, 1, 1.0),
    (12, 12, 4, 4, 1, 12, 0.3),
])
def test_plan_equals_brute_force(T, E, k, ep, tp, S, cf):
    rng = np.random.default_rng(T * 31 + E)
    logits = rng.standard_normal((T, E), dtype=np.float32)
    logits[:, 0] += 1.0   # some skew so that capacity binds
    idx, _ = oracle.route(logits, k)
    pl = oracle.plan(idx, E, ep, tp, S, cf)
    C = T if cf == 0 else min(T, math.ceil(cf * T * k / E))
    assert pl.C == C
    lists, kept_lists, final_order, stage_order, pos_final, pos_stage = brute_plan(idx, E, ep, tp, S, C)
    assert list(pl.counts) == [len(l) for l in lists]
    assert list(pl.kept) == [len(l) for l in kept_lists]
    assert list(pl.offsets) == [0] + list(np.cumsum([len(l) for l in kept_lists]))
    assert pl.R == len(final_order)
    np.testing.assert_array_equal(pl.pos_final, pos_final)
    np.testing.assert_array_equal(pl.pos_stage, pos_stage)
    U, Tu, E_loc = S * tp, T // (S * tp), E // ep
    for u in range(U):
        for e in range(E):
            blk = [p for p in kept_lists[e] if p[0] // Tu == u]
            assert pl.n[u, e] == len(blk)
            if blk:
                assert pl.stage_off[u, e] == pos_stage[blk[0]]
                assert pl.unit_base[u, e] == pos_final[blk[0]]
        for d in range(ep):
            assert pl.send_rows[u, d] == pl.n[u, d * E_loc:(d + 1) * E_loc].sum()
    assert pl.alive == int((pos_final >= 0).any(axis=1).sum())
    if cf > 0:
        assert (pos_final < 0).any(), "case was meant to exercise drops"


def test_plan_equals_brute_force_on_random_problems():
    rng = np.random.default_rng(77)
    for case in range(60):
        E = int(rng.integers(1, 20))
        k = int(rng.integers(1, min(E, 5) + 1))
        ep = int(rng.choice([d for d in range(1, E + 1) if E % d == 0]))
        tp, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        T = int(rng.integers(1, 30)) * tp * S
        cf = float(np.float32(rng.choice([0.0, 0.2, 0.5, 1.0, 1.7])))
        padded = int(rng.integers(0, 2))
        logits = rng.standard_normal((T, E), dtype=np.float32)
        if rng.integers(0, 2):
            logits = np.round(logits)                     # plenty of ties
        logits[:, 0] += np.float32(rng.choice([0.0, 1.0]))
        idx, _ = oracle.route(logits, k)
        for t in range(T):
            assert list(idx[t]) == brute_topk(logits[t], k)
        pl = oracle.plan(idx, E, ep, tp, S, cf, padded)
        C = T if cf == 0 else min(T, math.ceil(cf * T * k / E))
        lists, kept_lists, final_order, stage_order, pos_final, pos_stage = brute_plan(idx, E, ep, tp, S, C)
        assert pl.C == C and pl.R == len(final_order), case
        np.testing.assert_array_equal(pl.pos_stage, pos_stage)
        if padded:
            exp = -np.ones_like(pos_final)
            for e in range(E):
                for r, (t, j) in enumerate(kept_lists[e]):
                    exp[t, j] = e * C + r
            np.testing.assert_array_equal(pl.pos_final, exp)
            assert pl.final_rows == E * C
        else:
            np.testing.assert_array_equal(pl.pos_final, pos_final)
            assert pl.final_rows == pl.R


def test_plan_dropless_is_numpy_stable_argsort():
    rng = np.random.default_rng(5)
    T, E, k = 512, 16, 4
    idx, _ = oracle.route(rng.standard_normal((T, E), dtype=np.float32), k)
    pl = oracle.plan(idx, E, 4, 2, 4, 0.0)
    flat = idx.ravel().astype(np.int64)                 # pair p = t*k + j, token-major
    order = np.argsort(flat, kind="stable")             # FINAL row r holds pair order[r]
    np.testing.assert_array_equal(pl.counts, np.bincount(flat, minlength=E))
    np.testing.assert_array_equal(pl.offsets[1:], np.cumsum(np.bincount(flat, minlength=E)))
    inv = np.empty(T * k, np.int64)
    inv[order] = np.arange(T * k)
    np.testing.assert_array_equal(pl.pos_final.ravel(), inv)
    assert pl.R == T * k and pl.alive == T


def test_plan_invariants_with_drops():
    w = Workload("t", 4096, 8, FP32, 32, 4, 8, 4, 8, 1.0, zipf_s=1.2)
    logits = workloads.make_logits(w, seed=11)
    idx, _ = oracle.route(logits, w.top_k)
    pl = oracle.plan(idx, w.experts, w.ep, w.tp, w.slices, w.capacity_factor)
    T, k, E = w.tokens, w.top_k, w.experts
    assert pl.counts.sum() == T * k
    assert pl.kept.sum() == pl.R == pl.offsets[-1]
    assert (pl.kept == np.minimum(pl.counts, pl.C)).all()
    assert pl.R < T * k, "skew must cause drops here"
    for pos in (pl.pos_final, pl.pos_stage):
        live = pos[pos >= 0]
        assert live.size == pl.R
        assert np.array_equal(np.sort(live), np.arange(pl.R))      # bijection onto [0,R)
    assert ((pl.pos_final >= 0) == (pl.pos_stage >= 0)).all()
    # inside every expert segment of FINAL token indices strictly increase; segments in expert order
    tok = np.repeat(np.arange(T), k).reshape(T, k)
    row_tok = np.full(pl.R, -1)
    row_exp = np.full(pl.R, -1)
    m = pl.pos_final >= 0
    row_tok[pl.pos_final[m]] = tok[m]
    row_exp[pl.pos_final[m]] = idx[m]
    assert (np.diff(row_exp) >= 0).all()
    same = np.diff(row_exp) == 0
    assert (np.diff(row_tok)[same] > 0).all()
    # dropped pairs are exactly those whose rank among same-expert pairs (token order) is >= C
    for e in range(E):
        toks = np.sort(tok[idx == e])
        keep = set(toks[:pl.C].tolist())
        got = set(tok[(idx == e) & m].tolist())
        assert got == keep
    # in STAGE the key (unit, expert, token) is strictly increasing
    Tu = T // (w.slices * w.tp)
    s_tok = np.full(pl.R, -1)
    s_exp = np.full(pl.R, -1)
    s_tok[pl.pos_stage[m]] = tok[m]
    s_exp[pl.pos_stage[m]] = idx[m]
    key = (s_tok // Tu).astype(np.int64) * E * T + s_exp.astype(np.int64) * T + s_tok
    assert (np.diff(key) > 0).all()


# --------------------------------------------------------- pack / regather

@pytest.mark.parametrize("dtype", [FP32, BF16])
def test_pack_regather_against_explicit_gather(dtype):
    w = Workload("t", 96, 16, dtype, 6, 3, 3, 2, 4, 0.7)
    logits, x = workloads.make_inputs(w, seed=2)
    logits[:, 1] += 1.5
    r = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    C = oracle.capacity(w.tokens, w.experts, w.top_k, w.capacity_factor)
    _, _, final_order, stage_order, _, _ = brute_plan(r.topk_idx, w.experts, w.ep, w.tp, w.slices, C)
    np.testing.assert_array_equal(r.final, x[[t for t, _ in final_order]])
    np.testing.assert_array_equal(r.stage, x[[t for t, _ in stage_order]])
    assert r.final.dtype == x.dtype and r.stage.shape == (r.plan.R, w.hidden)


def test_pack_and_regather_slice_by_slice_equals_all_at_once():
    w = Workload("t", 120, 8, FP32, 4, 2, 2, 3, 4, 0.8)
    logits, x = workloads.make_inputs(w, seed=3)
    r = oracle.forward(logits, x, k=2, ep=2, tp=3, S=4, cf=0.8)
    stage = np.full_like(r.stage, 7)
    final = np.full_like(r.final, 9)
    for j in [2, 0, 3, 1]:                       # any order: slices are independent
        oracle.pack(x, r.plan, 3, 4, stage=stage, slice_=j)
        oracle.regather(stage, r.plan, 3, 4, final=final, slice_=j)
    np.testing.assert_array_equal(stage, r.stage)
    np.testing.assert_array_equal(final, r.final)
    # one slice alone touches exactly its own contiguous STAGE region and its own blocks of FINAL
    tp, S, E = 3, 4, 4
    Tu = 120 // (tp * S)
    for j in range(S):
        stage = np.full_like(r.stage, 7)
        final = np.full_like(r.final, 9)
        oracle.pack(x, r.plan, tp, S, stage=stage, slice_=j)
        oracle.regather(r.stage, r.plan, tp, S, final=final, slice_=j)
        m = r.plan.pos_stage >= 0
        tok = np.repeat(np.arange(120), 2).reshape(120, 2)
        in_slice = (tok // Tu) // tp == j
        rows_s = np.sort(r.plan.pos_stage[m & in_slice])
        assert rows_s.size and (np.diff(rows_s) == 1).all()          # the slice's region is contiguous
        touched = np.zeros(r.plan.R, bool)
        touched[rows_s] = True
        np.testing.assert_array_equal(stage[touched], r.stage[touched])
        assert (stage[~touched] == 7).all()
        touched_f = np.zeros(r.plan.R, bool)
        touched_f[r.plan.pos_final[m & in_slice]] = True
        np.testing.assert_array_equal(final[touched_f], r.final[touched_f])
        assert (final[~touched_f] == 9).all()


def test_tp_and_slices_do_not_change_the_result():
    """The paper's exactness claim: Drop + chunking + gather + D2D copy equals the plain AllToAll."""
    base = Workload("t", 240, 24, BF16, 8, 2, 4, 1, 1, 0.9)
    logits, x = workloads.make_inputs(base, seed=4)
    logits[:, 3] += 2.0
    ref = oracle.forward(logits, x, k=2, ep=4, tp=1, S=1, cf=0.9)
    assert (ref.plan.pos_final < 0).any()
    # with tp = S = 1 there is one unit: STAGE and FINAL coincide
    np.testing.assert_array_equal(ref.stage, ref.final)
    seen_different_stage = False
    for tp, S in itertools.product([1, 2, 3, 4], [1, 2, 5, 10]):
        if 240 % (tp * S):
            continue
        r = oracle.forward(logits, x, k=2, ep=4, tp=tp, S=S, cf=0.9)
        for a, b in [(r.topk_idx, ref.topk_idx), (r.gates, ref.gates), (r.plan.counts, ref.plan.counts),
                     (r.plan.kept, ref.plan.kept), (r.plan.offsets, ref.plan.offsets),
                     (r.plan.pos_final, ref.plan.pos_final), (r.final, ref.final), (r.out, ref.out)]:
            np.testing.assert_array_equal(a, b)
        seen_different_stage |= not np.array_equal(r.stage, ref.stage)
    assert seen_different_stage        # the intermediate really is laid out differently


# ------------------------------------------------------------------ combine

def test_round_trip_top1_is_exact():
    for dtype in (FP32, BF16):
        w = Workload("t", 128, 32, dtype, 4, 1, 2, 2, 2, 0.0)
        logits, x = workloads.make_inputs(w, seed=5)
        x[3, 7] = 0 if dtype == FP32 else 0x8000          # a negative zero (bf16) / zero
        if dtype == FP32:
            x[3, 8] = -0.0
        r = oracle.forward(logits, x, k=1, ep=2, tp=2, S=2, cf=0.0)
        assert (r.gates == 1.0).all()
        # exact as values; the sum starts from +0, so 0 + 1*(-0) = +0: a -0 input comes back as +0
        as_f = (lambda a: a) if dtype == FP32 else workloads.bf16_bits_to_f32
        np.testing.assert_array_equal(as_f(r.out), as_f(x))
        nz = as_f(x) != 0
        np.testing.assert_array_equal(r.out[nz], x[nz])


def test_round_trip_topk_renorm_returns_input():
    w = Workload("t", 128, 32, FP32, 8, 3, 2, 2, 2, 0.0)
    logits, x = workloads.make_inputs(w, seed=6)
    r = oracle.forward(logits, x, k=3, ep=2, tp=2, S=2, cf=0.0)
    assert np.all(np.abs(r.out.astype(np.float64) - x) <= 2 * ulp32(x))
    wb = w.with_(dtype=BF16)
    logits, xb = workloads.make_inputs(wb, seed=6)
    rb = oracle.forward(logits, xb, k=3, ep=2, tp=2, S=2, cf=0.0)
    d = np.abs(rb.out.astype(np.int32) - xb.astype(np.int32))      # neighbouring bf16 bit patterns
    assert d.max() <= 1


@pytest.mark.parametrize("dtype", [FP32, BF16])
@pytest.mark.parametrize("cf", [0.0, 0.6])
def test_combine_equals_dense_moe_definition(dtype, cf):
    """out[t] = sum_e G[t,e] * f_e(x[t]) with expert-specific f_e, no permutation anywhere."""
    w = Workload("t", 80, 12, dtype, 5, 2, 5, 2, 2, cf)
    logits, x = workloads.make_inputs(w, seed=8)
    logits[:, 2] += 1.0
    r = oracle.forward(logits, x, k=2, ep=5, tp=2, S=2, cf=cf, renorm=0)
    xf = x if dtype == FP32 else workloads.bf16_bits_to_f32(x)
    # expert e multiplies by (e+2)/4 : exact in fp32 and bf16 for bf16 inputs? keep it exact: powers of two
    scale = np.array([1.0, 0.5, 2.0, 0.25, 4.0])
    y = np.empty((r.plan.R, w.hidden), np.float32)
    for e in range(w.experts):
        seg = slice(r.plan.offsets[e], r.plan.offsets[e + 1])
        ff = r.final[seg] if dtype == FP32 else workloads.bf16_bits_to_f32(r.final[seg])
        y[seg] = ff * np.float32(scale[e])
    y_in = y if dtype == FP32 else workloads.f32_to_bf16_bits(y)   # exact: power-of-two scaling
    out = oracle.combine(y_in, r.gates, r.plan.pos_final)
    # dense definition
    C = oracle.capacity(w.tokens, w.experts, 2, cf)
    G = np.zeros((w.tokens, w.experts))
    seen = np.zeros(w.experts, int)
    for t in range(w.tokens):
        for j in range(2):
            e = r.topk_idx[t, j]
            if seen[e] < C:
                G[t, e] = float(r.gates[t, j])
        for j in range(2):
            seen[r.topk_idx[t, j]] += 1
    ref = np.zeros((w.tokens, w.hidden))
    for e in range(w.experts):
        ref += G[:, e:e + 1] * (xf.astype(np.float64) * scale[e])
    if cf > 0:
        assert (G.sum(1) == 0).any() or (r.plan.pos_final < 0).any()
    if dtype == FP32:
        assert np.all(np.abs(out.astype(np.float64) - ref) <= 0.5000001 * ulp32(ref) + 1e-300)
    else:
        import torch
        # the fp64 sums here are not fp32-exact, so allow the neighbouring bf16 value
        ref_bits = torch.tensor(ref, dtype=torch.float64).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.abs(out.astype(np.int32) - ref_bits.astype(np.int32)).max() <= 1
        back = workloads.bf16_bits_to_f32(out).astype(np.float64)
        assert np.all(np.abs(back - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-40)   # within half a bf16 ulp


def test_combine_bf16_rounding_is_nearest_even_single_rounding():
    import torch
    one, eps8, eps7 = 1.0, 2.0 ** -8, 2.0 ** -7
    cases = [
        ([one, eps8], 1.0),                      # exactly halfway between 1 and 1+2^-7: even mantissa wins
        ([one + eps7, eps8], 1.0 + 2 * eps7),    # halfway between odd and even: goes up to even
        ([one, eps8, 2.0 ** -16], 1.0 + eps7),  # just above halfway
        ([-one, -eps8], -1.0),
        ([3.0, 2.0 ** -7], 3.0),                 # halfway in [2,4): spacing 2^-6
        ([2.0 ** -130, 2.0 ** -133], None),      # subnormal bf16 range, checked against torch only
    ]
    for vals, expect in cases:
        m = len(vals)
        y = workloads.f32_to_bf16_bits(np.array(vals, np.float32).reshape(m, 1))
        assert np.array_equal(workloads.bf16_bits_to_f32(y).ravel(), np.array(vals, np.float32)), "inputs must be bf16-exact"
        gates = np.ones((1, m), np.float32)
        pos = np.arange(m, dtype=np.int32).reshape(1, m)
        out = oracle.combine(y, gates, pos)
        got = float(workloads.bf16_bits_to_f32(out)[0, 0])
        s = np.float32(sum(vals))                              # exact in fp32 for these inputs
        assert float(s) == sum(vals)
        tref = float(torch.tensor([s]).to(torch.bfloat16).to(torch.float32)[0])
        assert got == tref
        if expect is not None:
            assert got == expect
    # a double-rounding trap: sum = 1 + 2^-8 + 2^-30 is above halfway, but rounding to fp32 first
    # gives exactly halfway (1 + 2^-8) and then ties-to-even would give 1.0
    y = workloads.f32_to_bf16_bits(np.array([[1.0], [2.0 ** -8], [2.0 ** -30]], np.float32))
    out = oracle.combine(y, np.ones((1, 3), np.float32), np.array([[0, 1, 2]], np.int32))
    assert float(workloads.bf16_bits_to_f32(out)[0, 0]) == 1.0 + 2.0 ** -7


def test_combine_random_bf16_matches_torch_rounding_of_fp32_exact_sums():
    import torch
    rng = np.random.default_rng(9)
    R, H, T = 64, 40, 32
    # small-integer values and power-of-two gates: every partial sum is exact in fp32
    yv = rng.integers(-64, 64, size=(R, H)).astype(np.float32)
    y = workloads.f32_to_bf16_bits(yv)
    gates = (2.0 ** rng.integers(-6, 1, size=(T, 2))).astype(np.float32)
    pos = rng.permutation(R)[:T * 2].reshape(T, 2).astype(np.int32)
    pos[3, 1] = -1
    pos[5, :] = -1
    out = oracle.combine(y, gates, pos)
    acc = np.zeros((T, H), np.float32)
    for j in range(2):
        m = pos[:, j] >= 0
        acc[m] += gates[m, j:j + 1] * yv[pos[m, j]]
    ref = torch.tensor(acc).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(out, ref)
    assert (out[5] == 0).all()


def test_fully_dropped_token_gives_zero_row_and_gates_not_renormalised():
    logits = np.zeros((6, 2), np.float32)
    logits[:, 0] = 1.0                       # every token: expert 0 first, expert 1 second
    x = np.arange(6 * 4, dtype=np.float32).reshape(6, 4) + 1
    r = oracle.forward(logits, x, k=1, ep=1, tp=1, S=1, cf=1.0)   # C = ceil(1*6*1/2) = 3
    assert r.plan.C == 3 and r.plan.R == 3 and r.plan.alive == 3
    np.testing.assert_array_equal(r.out[:3], x[:3])
    assert (r.out[3:] == 0).all()
    r2 = oracle.forward(logits, x, k=2, ep=1, tp=1, S=1, cf=0.5)  # C = 3 again, both experts overflow
    g = r2.gates.astype(np.float64)
    np.testing.assert_allclose(r2.out[:3], (g[:3].sum(1, keepdims=True)) * x[:3], rtol=1e-6)
    assert (r2.out[3:] == 0).all()


def test_two_pass_gather_then_copy_equals_the_fused_pass():
    w = Workload("t", 180, 8, FP32, 5, 2, 5, 3, 4, 0.8)
    logits, x = workloads.make_inputs(w, seed=21)
    logits[:, 1] += 1.0
    r = oracle.forward(logits, x, k=2, ep=5, tp=3, S=4, cf=w.capacity_factor)
    g = np.full_like(r.stage, 3)
    for j in (3, 1, 0, 2):
        before = g.copy()
        oracle.allgather(r.stage, r.plan, 3, 4, gathered=g, slice_=j)
        a, b = r.plan.stage_off[j * 3, 0], (r.plan.stage_off[(j + 1) * 3, 0] if j < 3 else r.plan.R)
        np.testing.assert_array_equal(g[a:b], r.stage[a:b])          # exactly the slice's contiguous range
        np.testing.assert_array_equal(g[:a], before[:a])
        np.testing.assert_array_equal(g[b:], before[b:])
    np.testing.assert_array_equal(g, r.stage)
    np.testing.assert_array_equal(oracle.regather(g, r.plan, 3, 4), r.final)
    np.testing.assert_array_equal(oracle.allgather(r.stage, r.plan, 3, 4), r.stage)


@pytest.mark.parametrize("dtype", [FP32, BF16])
def test_padded_layout_is_the_capacity_tensor(dtype):
    w = Workload("t", 200, 16, dtype, 5, 2, 5, 2, 2, 0.8)
    logits, x = workloads.make_inputs(w, seed=31)
    logits[:, 0] += 1.5
    comp = oracle.forward(logits, x, k=2, ep=5, tp=2, S=2, cf=w.capacity_factor)
    padd = oracle.forward(logits, x, k=2, ep=5, tp=2, S=2, cf=w.capacity_factor, padded=1, fill=7)
    C, E = comp.plan.C, 5
    assert padd.plan.R == comp.plan.R and padd.plan.final_rows == E * C and padd.final.shape[0] == E * C
    assert list(padd.plan.offsets) == [e * C for e in range(E + 1)]
    cube = padd.final.reshape(E, C, w.hidden)
    for e in range(E):
        n_e = comp.plan.kept[e]
        np.testing.assert_array_equal(cube[e, :n_e], comp.final[comp.plan.offsets[e]:comp.plan.offsets[e + 1]])
        assert (cube[e, n_e:] == 0).all()                       # padding is zero-filled, not left at the fill value
    assert (comp.plan.kept < C).any() and (comp.plan.kept == C).any()
    # positions differ only by the segment base; STAGE is the same compact buffer; the result is the same
    m = comp.plan.pos_final >= 0
    e_of = comp.topk_idx[m]
    np.testing.assert_array_equal(padd.plan.pos_final[m] - e_of * C, comp.plan.pos_final[m] - comp.plan.offsets[e_of])
    np.testing.assert_array_equal(padd.plan.pos_final[~m], -1)
    np.testing.assert_array_equal(padd.stage, comp.stage)
    np.testing.assert_array_equal(padd.plan.pos_stage, comp.plan.pos_stage)
    np.testing.assert_array_equal(padd.out, comp.out)
    np.testing.assert_array_equal(padd.plan.unit_base - np.arange(E)[None, :] * C, comp.plan.unit_base - comp.plan.offsets[None, :E])
    # the return path works on it unchanged
    np.testing.assert_array_equal(oracle.unregather(padd.final, padd.plan, 2, 2), padd.stage)


# ------------------------------------------------------- mirrored return path

@pytest.mark.parametrize("dtype", [FP32, BF16])
def test_unregather_inverts_regather_and_staged_combine_equals_direct(dtype):
    w = Workload("t", 240, 24, dtype, 6, 3, 3, 4, 3, 0.7)
    logits, x = workloads.make_inputs(w, seed=12)
    logits[:, 4] += 1.5
    r = oracle.forward(logits, x, k=3, ep=3, tp=4, S=3, cf=0.7)
    assert (r.plan.pos_final < 0).any()
    # identity experts: the way back reproduces the send buffer exactly
    np.testing.assert_array_equal(oracle.unregather(r.final, r.plan, 4, 3), r.stage)
    # arbitrary expert output: explicit gather through the two position tables
    rng = np.random.default_rng(2)
    y = rng.standard_normal((r.plan.R, w.hidden), dtype=np.float32)
    if dtype == BF16:
        y = workloads.f32_to_bf16_bits(y)
    ys = oracle.unregather(y, r.plan, 4, 3, fill=0)
    m = r.plan.pos_final >= 0
    expect = np.zeros_like(y)
    expect[r.plan.pos_stage[m]] = y[r.plan.pos_final[m]]
    np.testing.assert_array_equal(ys, expect)
    # slice by slice, any order, only the slice's rows / tokens are touched
    ys2 = np.full_like(y, 7)
    out2 = np.full((w.tokens, w.hidden), 9, dtype=y.dtype)
    per_slice = w.tokens // 3
    for j in (1, 2, 0):
        oracle.unregather(y, r.plan, 4, 3, y_stage=ys2, slice_=j)
        oracle.combine_staged(ys2, r.gates, r.plan.pos_stage, out=out2, t0=j * per_slice, t1=(j + 1) * per_slice)
    np.testing.assert_array_equal(ys2, ys)
    # the mirrored path gives the very bits of the direct unpermutation (same sum, same order)
    direct = oracle.combine(y, r.gates, r.plan.pos_final)
    np.testing.assert_array_equal(out2, direct)
    np.testing.assert_array_equal(oracle.combine_staged(ys, r.gates, r.plan.pos_stage), direct)


# ------------------------------------------------------------------- volume

def read_table8():
    vals = {}
    with open(os.path.join(GOLDEN, "table8_volumes.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, b, v = line.split()
            vals[(a, b)] = int(v)
    return vals


def test_volume_matches_paper_table8():
    """Table 8's workload: 8K sequence, hidden 8192, t = 8, e = 2, 4 chunks, I = 256 M.

    I = b*s*h*BPE (Eq. 3) reaches 256 M with 4 bytes per element at b = 1 and one row per token."""
    M = 1 << 20
    tab = read_table8()
    T, H, bpe, E, k, ep, tp, S = 8192, 8192, 4, 2, 1, 2, 8, 4
    I = T * H * bpe
    assert I == tab[("baseline", "alltoall")] * M
    logits = workloads.make_logits(Workload("t", T, H, FP32, E, k, ep, tp, S, 0.0), seed=0)
    idx, _ = oracle.route(logits, k)
    pl = oracle.plan(idx, E, ep, tp, S, 0.0)
    unit_bytes, dest_bytes, slice_bytes = oracle.volume(pl, tp, S, H * bpe)
    assert unit_bytes.sum() == tab[("o1", "allgather")] * M               # gathered result = whole I
    per_rank = unit_bytes.reshape(S, tp).sum(0)
    assert (per_rank == tab[("o1", "alltoall")] * M).all()                # I / t
    assert (unit_bytes == tab[("chunked4", "alltoall_per_chunk")] * M).all()   # I / (N t)
    assert (slice_bytes == tab[("chunked4", "allgather_per_chunk")] * M).all()  # I / N
    assert (slice_bytes == tab[("chunked4", "d2d_per_chunk")] * M).all()
    assert (dest_bytes.sum(1) == unit_bytes).all()


@pytest.mark.parametrize("tp,S,k", [(1, 1, 1), (2, 4, 2), (8, 4, 1), (4, 8, 3)])
def test_volume_closed_form_split_cuts_traffic_by_tp(tp, S, k):
    T, H, E, ep = 1024, 64, 8, 4
    w = Workload("t", T, H, BF16, E, k, ep, tp, S, 0.0)
    idx, _ = oracle.route(workloads.make_logits(w, seed=1), k)
    pl = oracle.plan(idx, E, ep, tp, S, 0.0)
    unit_bytes, dest_bytes, slice_bytes = oracle.volume(pl, tp, S, w.row_bytes)
    I = T * w.row_bytes
    assert (unit_bytes == I * k // (S * tp)).all()       # every unit packs exactly Tu*k rows when nothing drops
    assert (slice_bytes == I * k // S).all()
    unsplit = oracle.volume(oracle.plan(idx, E, ep, 1, S, 0.0), 1, S, w.row_bytes)[0]
    assert (unit_bytes.reshape(S, tp).sum(1) == unsplit).all()
    assert (unit_bytes.reshape(S, tp)[:, 0] * tp == unsplit).all()     # exactly 1/tp per TP rank


def test_volume_with_drops_counts_rows_per_slice():
    w = Workload("t", 600, 8, BF16, 6, 2, 3, 2, 5, 0.5, zipf_s=1.0)
    idx, _ = oracle.route(workloads.make_logits(w, seed=2), 2)
    pl = oracle.plan(idx, 6, 3, 2, 5, 0.5)
    unit_bytes, dest_bytes, slice_bytes = oracle.volume(pl, 2, 5, w.row_bytes)
    Tu = 600 // 10
    tok = np.repeat(np.arange(600), 2).reshape(600, 2)
    m = pl.pos_final >= 0
    per_slice = np.bincount((tok[m] // Tu) // 2, minlength=5) * w.row_bytes
    per_unit = np.bincount(tok[m] // Tu, minlength=10) * w.row_bytes
    assert len(set(per_slice.tolist())) > 1, "drops must make the slices uneven"
    np.testing.assert_array_equal(slice_bytes, per_slice)
    np.testing.assert_array_equal(unit_bytes, per_unit)
    for d in range(3):
        md = m & (idx // 2 == d)
        np.testing.assert_array_equal(dest_bytes[:, d], np.bincount(tok[md] // Tu, minlength=10) * w.row_bytes)


def test_off_rank_fraction_is_about_e_minus_1_over_e():
    # Eq. 8's (e-1)/e factor: with uniform routing a share 1/ep of the rows stays on the sender's EP rank
    w = workloads.CONFIGS["2x70b"]
    idx, _ = oracle.route(workloads.make_logits(w), w.top_k)
    pl = oracle.plan(idx, w.experts, w.ep, w.tp, w.slices, 0.0)
    rows = pl.send_rows.sum(0)
    assert rows.sum() == w.tokens
    frac_off = 1.0 - rows[0] / rows.sum()
    assert abs(frac_off - (w.ep - 1) / w.ep) < 0.02


# ------------------------------------------------- workload fingerprints

def numpy_fingerprint(w):
    logits = workloads.make_logits(w)
    order = np.argsort(-logits, axis=1, kind="stable")[:, :w.top_k]
    counts = np.bincount(order.ravel(), minlength=w.experts)
    C = w.tokens if w.capacity_factor == 0 else min(w.tokens, math.ceil(w.capacity_factor * w.tokens * w.top_k / w.experts))
    return order, counts, C


@pytest.mark.parametrize("name", ["mixtral", "2x70b", "longctx", "skewed"])
def test_named_workloads_route_and_plan_at_full_size(name):
    w = workloads.CONFIGS[name]
    order, counts, C = numpy_fingerprint(w)
    logits = workloads.make_logits(w)
    idx, gates = oracle.route(logits, w.top_k)
    np.testing.assert_array_equal(idx, order)
    pl = oracle.plan(idx, w.experts, w.ep, w.tp, w.slices, w.capacity_factor)
    np.testing.assert_array_equal(pl.counts, counts)
    assert pl.C == C and pl.R == int(np.minimum(counts, C).sum())
    # alive tokens by a vectorised rank computation: rank of a pair = position among equal experts (stable)
    flat = order.ravel()
    srt = np.argsort(flat, kind="stable")
    starts = np.concatenate([[0], np.cumsum(counts)])[:-1]
    rank = np.empty(flat.size, np.int64)
    rank[srt] = np.arange(flat.size) - np.repeat(starts, counts)
    assert pl.alive == int((rank.reshape(order.shape) < C).any(axis=1).sum())
    expect = {"mixtral": (16384, 2101), "2x70b": (8192, 4104), "longctx": (65536, 8309), "skewed": (233178, 64541)}[name]
    assert (pl.R, int(counts.max())) == expect
    if name == "skewed":
        assert pl.alive == 63030 and int(counts.min()) == 146
        assert list(pl.send_rows.sum(0)) == [81920, 78017, 38625, 16924, 8621, 4700, 2721, 1650]


# ------------------------------------------------------------ the all-cores timing build

@pytest.mark.parametrize("dtype,cf,padded", [(BF16, 0.6, 0), (FP32, 0.0, 0), (BF16, 1.25, 1)])
def test_openmp_build_gives_the_same_bytes_as_the_plain_build(dtype, cf, padded):
    """The -fopenmp build of the same source (used only to time the CPU baseline on every core) deals
    independent iterations to threads: every array it produces must equal the single-threaded build's."""
    w = Workload("omp", 1536, 264, dtype, 12, 3, 4, 2, 3, cf, zipf_s=0.9, padded=padded)
    logits, x = workloads.make_inputs(w, seed=11)
    kw = dict(k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor, padded=padded)
    assert oracle.threads() == 1
    a = oracle.forward(logits, x, **kw)
    with oracle.all_cores():
        assert oracle.threads() >= 1
        b = oracle.forward(logits, x, **kw)
        c = oracle.forward(logits, x, reuse=b, **kw)        # written again in place: the timing loop's form
    assert oracle.threads() == 1
    for r in (b, c):
        for f in ("topk_idx", "gates", "stage", "final", "out"):
            assert np.array_equal(getattr(a, f).view(np.uint8), getattr(r, f).view(np.uint8)), f
        for f in ("counts", "kept", "offsets", "pos_final", "pos_stage", "n", "stage_off", "unit_base", "send_rows"):
            assert np.array_equal(getattr(a.plan, f), getattr(r.plan, f)), f
