"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.

Bar: bit-exact on indices, every plan table, STAGE and FINAL (rows past R must keep
their canary); gates within 1e-6 relative (both sides evaluate them in fp64 and
round once; only the exp() implementations differ); combine within
1e-6 * sum_j |g_j*y_j| per element for fp32 and within 1e-2 absolute for bf16.
The kernel carries the combine sum in fp64 in the oracle's order, so wherever the
two sides' gates are bitwise equal the output must be bitwise equal as well; that
stronger check is applied to every such token.
"""
import sys

import numpy as np
import pytest

import oracle
import workloads
from workloads import BF16, FP32, Workload

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def m():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_00662_amd as mod
    mod.binding.lib()          # fails loudly if the HIP library is not built
    return mod


def cfg_of(m, w: Workload):
    return m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm,
                      w.padded)


def run_gpu(m, w, logits, x, mode=1, how="pipeline", canary=0xA5, repeats=1, plan_mode=-1, cache=-1):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    cfg = cfg_of(m, w)
    b = m.alloc_buffers(cfg, logits, x, canary=canary)
    m.monta_set_pipeline_mode(mode)
    m.monta_set_plan_mode(plan_mode)
    m.monta_set_cache_policy(cache)
    for _ in range(repeats):
        if how == "fused_call":
            m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
            m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
            continue
        m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
        if how == "pipeline":
            m.monta_dispatch_regather(cfg, b.x, b.stage, b.final, b.ws)
        elif how == "all":
            m.monta_dispatch(cfg, b.x, b.stage, b.ws, -1)
            m.monta_regather(cfg, b.stage, b.final, b.ws, -1)
        elif how == "slices_reversed":
            for j in reversed(range(w.slices)):
                m.monta_dispatch(cfg, b.x, b.stage, b.ws, j)
            for j in reversed(range(w.slices)):
                m.monta_regather(cfg, b.stage, b.final, b.ws, j)
        else:
            raise ValueError(how)
        m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
    torch.cuda.synchronize()
    m.monta_set_pipeline_mode(-1)
    m.monta_set_plan_mode(-1)
    m.monta_set_cache_policy(-1)
    tabs = m.read_tables(cfg, b.ws)
    res = dict(tabs)
    res["topk_idx"] = b.topk_idx.cpu().numpy()
    res["gates"] = b.gates.cpu().numpy()
    res["stage_full"] = bufs.to_host_act(cfg, b.stage)
    res["final_full"] = bufs.to_host_act(cfg, b.final)
    res["out"] = bufs.to_host_act(cfg, b.out)
    res["buffers"] = b
    return res


def canary_value(dtype, byte=0xA5):
    return np.frombuffer(bytes([byte] * 4), dtype=np.float32)[0] if dtype == FP32 else np.uint16(byte * 257)


def check_against_oracle(w, logits, x, got, ref=None, canary=0xA5):
    if ref is None:
        ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor, renorm=w.renorm,
                             padded=w.padded, fill=canary if canary is not None else 0)
    pl = ref.plan
    np.testing.assert_array_equal(got["topk_idx"], ref.topk_idx)
    g, gr = got["gates"].astype(np.float64), ref.gates.astype(np.float64)
    assert np.all(np.abs(g - gr) <= 1e-6 * np.abs(gr)), f"gates: max rel {np.max(np.abs(g - gr) / np.abs(gr))}"
    assert got["R"] == pl.R and got["alive"] == pl.alive and got["C"] == pl.C and got["final_rows"] == pl.final_rows
    for name in ["counts", "kept", "offsets", "n", "stage_off", "unit_base", "send_rows", "pos_final", "pos_stage"]:
        np.testing.assert_array_equal(got[name], getattr(pl, name), err_msg=name)
    U = w.slices * w.tp
    np.testing.assert_array_equal(got["unit_rows"][:U], pl.stage_off[:, 0])
    assert got["unit_rows"][U] == pl.R
    np.testing.assert_array_equal(got["kept_prefix"], np.concatenate([[0], np.cumsum(pl.kept)]))
    # STAGE -> FINAL row map, from the oracle's two position tables
    rm = np.full(pl.R, -1, np.int32)
    live = pl.pos_stage >= 0
    rm[pl.pos_stage[live]] = pl.pos_final[live]
    np.testing.assert_array_equal(got["row_map"][:pl.R], rm)
    # buffers: bit-exact below R, untouched above
    for name, refbuf, rows in (("stage_full", ref.stage, pl.R), ("final_full", ref.final, pl.final_rows)):
        buf = got[name]
        assert buf.dtype == refbuf.dtype
        np.testing.assert_array_equal(buf[:rows], refbuf, err_msg=name)
        if canary is not None and buf.shape[0] > rows:
            tail = buf[rows:]
            assert (tail.view(np.uint8) == canary).all(), f"{name}: rows past the end were written"
    check_combine(w, got["out"], ref.out, ref.final, ref.gates, pl.pos_final, got["gates"])
    return ref


def check_combine(w, out, ref_out, y, gates, pos_final, gpu_gates):
    k = w.top_k
    same = (gpu_gates.view(np.uint32) == gates.view(np.uint32)).all(axis=1)
    assert same.mean() > 0.99, "gates should be bitwise equal for nearly every token"
    np.testing.assert_array_equal(out[same], ref_out[same], err_msg="combine: same gates must give the same bits")
    if w.dtype == FP32:
        absum = np.zeros(out.shape, np.float64)
        for j in range(k):
            mj = pos_final[:, j] >= 0
            absum[mj] += np.abs(gates[mj, j:j + 1].astype(np.float64) * y[pos_final[mj, j]])
        tol = 1e-6 * absum + 1e-37
        d = np.abs(out.astype(np.float64) - ref_out.astype(np.float64))
        assert np.all(d <= tol), f"combine fp32: worst ratio {np.max(d / tol)}"
    else:
        a = workloads.bf16_bits_to_f32(out).astype(np.float64)
        r = workloads.bf16_bits_to_f32(ref_out).astype(np.float64)
        d = np.abs(a - r)
        assert d.max() <= 1e-2, f"combine bf16: max abs diff {d.max()}"
    dead = ~(pos_final >= 0).any(axis=1)
    if dead.any():
        assert (out[dead] == 0).all()


# ------------------------------------------------------------ named workloads

def test_tiny_all_modes(m):
    w = workloads.CONFIGS["tiny"]
    logits, x = workloads.make_inputs(w)
    ref = None
    for mode in (0, 1, 2):
        for how in ("pipeline", "all", "slices_reversed", "fused_call"):
            for plan_mode in (-1, 0):
                _say(f"tiny mode={mode} how={how} plan_mode={plan_mode}")
                got = run_gpu(m, w, logits, x, mode=mode, how=how, plan_mode=plan_mode)
                ref = check_against_oracle(w, logits, x, got, ref)
    # identity experts and renormalised gates: the input comes back
    assert np.all(np.abs(got["out"].astype(np.float64) - x) <= 2 * np.spacing(np.abs(x)))


@pytest.mark.parametrize("name", ["mixtral", "2x70b"])
@pytest.mark.parametrize("seed", [0, 1])
def test_named_8k_workloads(m, name, seed):
    w = workloads.CONFIGS[name]
    logits, x = workloads.make_inputs(w, seed=seed)
    _say(f"{name} seed={seed} oracle")
    ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    for mode in ((0, 1, 2) if seed == 0 else (1,)):
        _say(f"{name} seed={seed} mode={mode} gpu")
        got = run_gpu(m, w, logits, x, mode=mode, repeats=2, plan_mode=-1 if mode != 2 else 0)
        check_against_oracle(w, logits, x, got, ref)
    for cache in (0, 63, 21, 42):            # every stream cacheable / streaming / mixed
        _say(f"{name} seed={seed} cache={cache} gpu")
        got = run_gpu(m, w, logits, x, mode=1, cache=cache, how="fused_call" if cache in (0, 21) else "pipeline")
        check_against_oracle(w, logits, x, got, ref)
    _say(f"{name} seed={seed} fused call, twice")
    got = run_gpu(m, w, logits, x, mode=-1, how="fused_call", repeats=2)      # the calls and the mode bench.py times
    check_against_oracle(w, logits, x, got, ref)
    if name == "2x70b":
        # top-1, gate 1.0: exact round trip (as values: 0 + 1*(-0) is +0, so a -0 input comes back as +0)
        np.testing.assert_array_equal(workloads.bf16_bits_to_f32(got["out"]), workloads.bf16_bits_to_f32(x))


def test_longctx_slice_sweep(m):
    base = workloads.CONFIGS["longctx"]
    logits, x = workloads.make_inputs(base)
    ref1 = None
    for S in (1, 2, 4, 8):
        w = base.with_(slices=S)
        _say(f"longctx S={S} oracle")
        idx, gates = (ref1.topk_idx, ref1.gates) if ref1 else oracle.route(logits, w.top_k)
        pl = oracle.plan(idx, w.experts, w.ep, w.tp, S, w.capacity_factor)
        stage = oracle.pack(x, pl, w.tp, S)
        if ref1 is None:
            final = oracle.regather(stage, pl, w.tp, S)
            out = oracle.combine(final, gates, pl.pos_final)
            ref1 = oracle.Result(idx, gates, pl, stage, final, out)
            ref = ref1
        else:
            ref = oracle.Result(idx, gates, pl, stage, ref1.final, ref1.out)    # FINAL and out do not depend on S
            np.testing.assert_array_equal(pl.pos_final, ref1.plan.pos_final)
        for mode in ((0, 1, -1) if S in (1, 4) else (1, -1)):
            _say(f"longctx S={S} mode={mode} gpu")
            got = run_gpu(m, w, logits, x, mode=mode, how="fused_call" if mode in (1, -1) else "pipeline")
            check_against_oracle(w, logits, x, got, ref)
        del stage


def test_skewed_full_size(m):
    w = workloads.CONFIGS["skewed"]
    logits, x = workloads.make_inputs(w)
    _say("skewed oracle")
    ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    assert ref.plan.R == 233178 and ref.plan.alive == 63030
    _say("skewed gpu, default mode, the calls bench.py times")
    got = run_gpu(m, w, logits, x, mode=-1, how="fused_call")
    # full buffers are 7 GiB each on the host: compare the live part, then the canary on a sample of the tail
    R = ref.plan.R
    for name in ("stage_full", "final_full"):
        tail = got[name][R:]
        step = max(1, tail.shape[0] // 4096)
        assert (tail[::step].view(np.uint8) == 0xA5).all()
        assert (tail[:64].view(np.uint8) == 0xA5).all()
        got[name] = got[name][:R]
    check_against_oracle(w, logits, x, got, ref, canary=None)
    got.clear()
    _say("skewed gpu mode 0, ticketed plan")
    got = run_gpu(m, w, logits, x, mode=0, plan_mode=0)
    for name in ("stage_full", "final_full"):
        got[name] = got[name][:R]
    check_against_oracle(w, logits, x, got, ref, canary=None)


# ------------------------------------------------------- shapes and edge cases

EDGE = [
    # T, H, dtype, E, k, ep, tp, S, cf, renorm
    (1, 4, FP32, 1, 1, 1, 1, 1, 0.0, 1),            # the smallest problem: one 16-byte row
    (6, 8, BF16, 2, 2, 2, 3, 2, 0.0, 1),            # one token per unit, k = E
    (70, 12, FP32, 3, 2, 1, 1, 1, 0.0, 0),          # ragged route workgroup, row of 3 vectors, no renorm
    (330, 40, BF16, 5, 3, 5, 2, 3, 0.7, 1),         # Tu = 55, drops
    (1000, 264, BF16, 7, 7, 7, 5, 2, 0.5, 0),       # Tu = 100, k = E, 33 vectors per row, heavy drops
    (777, 100, FP32, 256, 32, 16, 7, 3, 0.9, 1),    # the limits: E = 256, k = 32; Tu = 37
    (4096, 1028, FP32, 16, 4, 4, 2, 2, 0.3, 1),     # 257 vectors per row: ragged second pass of the movers
    (5120, 2056, BF16, 64, 6, 8, 4, 5, 1.0, 1),     # 257 vectors, Tu = 256
    (2048, 7168, BF16, 32, 8, 8, 4, 4, 0.25, 1),    # 896 vectors: 3.5 passes of 256 lanes
    (600, 64, BF16, 8, 2, 4, 1, 1, 0.01, 1),        # capacity 2: almost everything dropped
    (4096, 8, BF16, 32, 2, 4, 64, 64, 0.9, 1),      # 4096 one-token units: histogram table too large for the
                                                    # per-workgroup rebuild, the ticketed scan takes over
]


@pytest.mark.parametrize("T,H,dtype,E,k,ep,tp,S,cf,renorm", EDGE)
def test_edge_shapes(m, T, H, dtype, E, k, ep, tp, S, cf, renorm):
    w = Workload("edge", T, H, dtype, E, k, ep, tp, S, cf, renorm=renorm, zipf_s=0.8 if cf > 0 else 0.0)
    logits, x = workloads.make_inputs(w, seed=T + E)
    ref = None
    for mode in (0, 1, 2):
        _say(f"edge {T},{H},{dtype},{E},{k},{ep},{tp},{S},{cf},{renorm} mode={mode}")
        got = run_gpu(m, w, logits, x, mode=mode, plan_mode=-1 if mode != 2 else 0)
        ref = check_against_oracle(w, logits, x, got, ref)
    _say(f"edge {T},{H},{dtype},{E},{k},{ep},{tp},{S},{cf},{renorm} fused call")
    got = run_gpu(m, w, logits, x, mode=1, how="fused_call")
    check_against_oracle(w, logits, x, got, ref)
    if cf > 0:
        assert (ref.plan.pos_final < 0).any()


def test_tied_logits_resolve_to_lower_index(m):
    w = Workload("ties", 512, 32, FP32, 16, 4, 4, 2, 2, 0.0)
    logits = workloads.make_tied_logits(w, levels=3, seed=5)
    _, x = workloads.make_inputs(w, seed=5)
    got = run_gpu(m, w, logits, x)
    check_against_oracle(w, logits, x, got)
    const = np.zeros_like(logits)                       # every logit equal: experts 0..k-1 win
    got = run_gpu(m, w, const, x)
    assert (got["topk_idx"] == np.arange(4)[None, :]).all()
    check_against_oracle(w, const, x, got)


def test_tp_and_slices_leave_final_and_out_unchanged(m):
    base = Workload("indep", 960, 256, BF16, 8, 2, 4, 1, 1, 0.8, zipf_s=1.0)
    logits, x = workloads.make_inputs(base, seed=3)
    first = None
    stages = []
    for tp, S in [(1, 1), (2, 1), (1, 4), (4, 3), (8, 5), (3, 8)]:
        w = base.with_(tp=tp, slices=S)
        got = run_gpu(m, w, logits, x)
        R = got["R"]
        if first is None:
            first = got
            np.testing.assert_array_equal(got["stage_full"][:R], got["final_full"][:R])
        for name in ("topk_idx", "gates", "counts", "kept", "offsets", "pos_final", "out"):
            np.testing.assert_array_equal(got[name], first[name], err_msg=f"{name} tp={tp} S={S}")
        np.testing.assert_array_equal(got["final_full"][:R], first["final_full"][:R])
        stages.append(got["stage_full"][:R].copy())
    assert any(not np.array_equal(s, stages[0]) for s in stages[1:])


def test_non_identity_experts_and_shared_gates(m):
    """Combine alone, both sides fed the same gates and the same expert output y != FINAL."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    for dtype in (FP32, BF16):
        w = Workload("y", 1024, 512, dtype, 8, 4, 4, 2, 2, 0.6, zipf_s=1.0)
        logits, x = workloads.make_inputs(w, seed=9)
        ref = oracle.forward(logits, x, k=4, ep=4, tp=2, S=2, cf=w.capacity_factor)
        rng = np.random.default_rng(1)
        y = rng.standard_normal((ref.plan.R, w.hidden), dtype=np.float32) * 3
        if dtype == BF16:
            y = workloads.f32_to_bf16_bits(y)
        ref_out = oracle.combine(y, ref.gates, ref.plan.pos_final)
        cfg = cfg_of(m, w)
        b = m.alloc_buffers(cfg, logits, x, canary=0)
        m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
        b.gates.copy_(torch.from_numpy(ref.gates).cuda())
        ydev = bufs.to_device_act(cfg, y)
        b.final[:ref.plan.R].copy_(ydev)
        m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
        torch.cuda.synchronize()
        out = bufs.to_host_act(cfg, b.out)
        check_combine(w, out, ref_out, y, ref.gates, ref.plan.pos_final, ref.gates)
        np.testing.assert_array_equal(out, ref_out)


def test_combine_rounding_traps_at_bf16_midpoints(m):
    """Sums that sit exactly on, or a hair beside, the midpoint between two bf16 values: rounding the fp64 sum
    to fp32 first lands exactly on the midpoint, so a kernel that then rounded to nearest-even again would go
    the wrong way.  Expected values follow from the construction (closed form), and the oracle must agree."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    T, H, E, k = 512, 256, 4, 2
    w = Workload("traps", T, H, BF16, E, k, 2, 2, 2, 0.0)
    logits, x = workloads.make_inputs(w, seed=4)
    ref = oracle.forward(logits, x, k=k, ep=2, tp=2, S=2, cf=0.0)
    R = ref.plan.R
    assert R == T * k
    rng = np.random.default_rng(7)
    # token t: out = g0 * 1.0 + g1 * y1 with g0 = a bf16 midpoint (9 significant bits, exact in fp32) and
    # g1 * y1 = 0 (true tie), or +/- a term far below fp32 resolution of the sum (the trap)
    mant = rng.integers(0, 128, size=T)                       # bf16 mantissa of the lower neighbour
    expo = rng.integers(-6, 7, size=T)
    sign = rng.choice([-1.0, 1.0], size=T)
    lower = (1.0 + mant / 128.0) * 2.0 ** expo                # a bf16 value
    mid = lower + 2.0 ** (expo - 8.0)                         # halfway to the next one
    kind = rng.integers(0, 3, size=T)                         # 0 tie, 1 just above, 2 just below
    tiny = np.float32(2.0 ** -40)
    gates = np.zeros((T, k), np.float32)
    gates[:, 0] = (sign * mid).astype(np.float32)
    assert np.array_equal(gates[:, 0].astype(np.float64), sign * mid)
    gates[:, 1] = np.where(kind == 0, 0.0, tiny * 2.0 ** expo).astype(np.float32)
    y = np.zeros((R, H), np.float32)
    pf = ref.plan.pos_final
    y[pf[:, 0]] = 1.0
    y[pf[:, 1]] = (np.where(kind == 1, 1.0, -1.0) * sign)[:, None]
    ybits = workloads.f32_to_bf16_bits(y)
    up = lower + 2.0 ** (expo - 7.0)
    even_is_lower = (mant % 2 == 0)
    want = np.where(kind == 1, up, np.where(kind == 2, lower, np.where(even_is_lower, lower, up))) * sign
    want_bits = workloads.f32_to_bf16_bits(np.repeat(want.astype(np.float32)[:, None], H, axis=1))
    ref_out = oracle.combine(ybits, gates, pf)
    np.testing.assert_array_equal(ref_out, want_bits)          # the oracle against the closed form
    cfg = cfg_of(m, w)
    b = m.alloc_buffers(cfg, logits, x, canary=0)
    m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
    b.gates.copy_(torch.from_numpy(gates).cuda())
    b.final[:R].copy_(bufs.to_device_act(cfg, ybits))
    m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bufs.to_host_act(cfg, b.out), want_bits)


def test_workspace_reuse_across_different_inputs(m):
    """The ticket counter and every table must be rebuilt on each call."""
    import torch
    w = Workload("reuse", 2048, 128, BF16, 8, 2, 2, 2, 4, 0.9, zipf_s=0.5)
    cfg = cfg_of(m, w)
    b = None
    for seed in (1, 2, 3):
        logits, x = workloads.make_inputs(w, seed=seed)
        if b is None:
            b = m.alloc_buffers(cfg, logits, x, canary=0)
        else:
            b.logits.copy_(torch.from_numpy(logits).cuda())
            b.x.copy_(torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16))
        m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
        m.monta_dispatch_regather(cfg, b.x, b.stage, b.final, b.ws)
        m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
        torch.cuda.synchronize()
        ref = oracle.forward(logits, x, k=2, ep=2, tp=2, S=4, cf=w.capacity_factor)
        tabs = m.read_tables(cfg, b.ws)
        assert tabs["R"] == ref.plan.R and tabs["alive"] == ref.plan.alive
        np.testing.assert_array_equal(tabs["pos_stage"], ref.plan.pos_stage)
        from paper_2411_00662_amd import buffers as bufs
        np.testing.assert_array_equal(bufs.to_host_act(cfg, b.final, ref.plan.R), ref.final)
        np.testing.assert_array_equal(b.topk_idx.cpu().numpy(), ref.topk_idx)


def test_copy_kernel_and_profile_counters(m):
    import torch
    n = (1 << 20) + 48
    src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    m.monta_profile_reset()
    m.monta_profile_enable(True)
    m.monta_copy(dst, src, n)
    m.monta_copy(dst, src, n)
    m.monta_profile_enable(False)
    ms, launches = m.monta_profile_read(6)
    torch.cuda.synchronize()
    assert launches == 2 and ms > 0
    assert torch.equal(dst, src)
    m.monta_profile_reset()
    assert m.monta_profile_read(6) == (0.0, 0)


def test_hip_graph_replays_match_eager(m):
    """The step captured in a HIP graph (no memset nodes: the library clears its counters in kernels) and
    replayed several times, with eager work and synchronisations in between, gives the eager bits every time."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w = Workload("graph", 4096, 1024, BF16, 8, 2, 4, 2, 4, 0.8, zipf_s=0.6)
    cfg = cfg_of(m, w)
    m.monta_set_pipeline_mode(-1)        # the default: launch groups chosen by size (three launches here)
    inputs = [workloads.make_inputs(w, seed=s) for s in (1, 2, 3)]
    b = m.alloc_buffers(cfg, *inputs[0], canary=0)
    stream = torch.cuda.Stream()

    def step():
        m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws, stream)
        m.monta_combine(cfg, b.final, b.gates, b.out, b.ws, stream)

    def snapshot():
        torch.cuda.synchronize()
        tabs = m.read_tables(cfg, b.ws)
        return (tabs["R"], tabs["alive"], tabs["pos_final"].copy(), tabs["pos_stage"].copy(), b.topk_idx.cpu().numpy(),
                bufs.to_host_act(cfg, b.final, tabs["R"]).copy(), bufs.to_host_act(cfg, b.out).copy())

    def load(i):
        logits, x = inputs[i]
        b.logits.copy_(torch.from_numpy(logits).cuda())
        b.x.copy_(torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16))
        torch.cuda.synchronize()

    eager = []
    for i in range(3):
        load(i)
        with torch.cuda.stream(stream):
            step()
        eager.append(snapshot())
    load(0)
    with torch.cuda.stream(stream):
        step()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
    for rep in range(2):
        for i in (2, 0, 1):
            _say(f"graph replay rep={rep} input={i}")
            load(i)
            b.out.zero_()
            b.final.zero_()
            graph.replay()
            got = snapshot()
            for a, e in zip(got, eager[i]):
                np.testing.assert_array_equal(a, e)
            with torch.cuda.stream(stream):          # eager work between the replays
                step()
            for a, e in zip(snapshot(), eager[i]):
                np.testing.assert_array_equal(a, e)
    ref = oracle.forward(*inputs[1], k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    assert eager[1][0] == ref.plan.R and np.array_equal(eager[1][5], ref.final)


def test_random_small_shapes(m):
    """Seeded random problems: every entry-point combination must agree with the oracle on each."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 40:
        E = int(rng.integers(1, 49))
        k = int(rng.integers(1, min(E, 6) + 1))
        ep = int(rng.choice([d for d in range(1, E + 1) if E % d == 0]))
        tp, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        Tu = int(rng.integers(1, 300))
        T = Tu * tp * S
        dtype = int(rng.integers(0, 2))
        H = int(rng.integers(1, 80)) * (4 if dtype == FP32 else 8)
        cf = float(rng.choice([0.0, 0.3, 0.75, 1.0, 1.5]))
        renorm = int(rng.integers(0, 2))
        w = Workload("rand", T, H, dtype, E, k, ep, tp, S, cf, renorm=renorm, zipf_s=float(rng.choice([0.0, 0.7])))
        logits, x = workloads.make_inputs(w, seed=1000 + done)
        mode = int(rng.integers(-1, 3))          # -1: the size-chosen launch grouping
        how = str(rng.choice(["pipeline", "all", "slices_reversed", "fused_call"]))
        plan_mode = int(rng.choice([-1, 0]))
        cache = int(rng.integers(-1, 64))
        _say(f"random {done}: T={T} H={H} dtype={dtype} E={E} k={k} ep={ep} tp={tp} S={S} cf={cf} renorm={renorm} "
             f"mode={mode} how={how} plan_mode={plan_mode} cache={cache}")
        got = run_gpu(m, w, logits, x, mode=mode, how=how, plan_mode=plan_mode, cache=cache)
        check_against_oracle(w, logits, x, got)
        done += 1


PADDED = [
    Workload("p1", 330, 40, BF16, 5, 3, 5, 2, 3, 0.7, zipf_s=0.8, padded=1),
    Workload("p2", 4096, 1028, FP32, 16, 4, 4, 2, 2, 0.3, zipf_s=0.8, padded=1),
    Workload("p3", 1000, 264, BF16, 7, 7, 7, 5, 2, 0.5, renorm=0, zipf_s=0.8, padded=1),
    Workload("p4", 600, 64, BF16, 8, 2, 4, 1, 1, 0.0, padded=1),                       # cf = 0: C = T, huge padding
    Workload("p5", 4096, 8, BF16, 32, 2, 4, 64, 64, 0.9, zipf_s=0.8, padded=1),        # ticketed plan path
    workloads.CONFIGS["mixtral"].with_(padded=1),
    workloads.CONFIGS["longctx"].with_(padded=1, tokens=8192),
]


@pytest.mark.parametrize("w", PADDED, ids=lambda w: w.name + "-padded")
def test_padded_layout(m, w):
    """FINAL as the capacity tensor [E][C][H]: kept rows first in every expert segment, zero padding after them."""
    logits, x = workloads.make_inputs(w, seed=7)
    ref = None
    for mode, how, plan_mode in ((1, "fused_call", -1), (0, "pipeline", -1), (2, "all", 0), (1, "slices_reversed", -1)):
        _say(f"padded {w.name} mode={mode} how={how} plan_mode={plan_mode}")
        got = run_gpu(m, w, logits, x, mode=mode, how=how, plan_mode=plan_mode)
        ref = check_against_oracle(w, logits, x, got, ref)
    C, E = ref.plan.C, w.experts
    assert got["final_full"].shape[0] == E * C == ref.plan.final_rows
    cube = got["final_full"].reshape(E, C, w.hidden)
    for e in range(E):
        assert (cube[e, ref.plan.kept[e]:] == 0).all()
    # same result as the compact layout
    wc = w.with_(padded=0)
    gotc = run_gpu(m, wc, logits, x, mode=1, how="fused_call")
    np.testing.assert_array_equal(gotc["out"], got["out"])
    np.testing.assert_array_equal(gotc["stage_full"][:ref.plan.R], got["stage_full"][:ref.plan.R])
