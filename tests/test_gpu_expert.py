"""GPU parity of the expert layer (monta_expert_linear, a grouped GEMM over the expert-major buffer).

Bar.  The oracle sums x[r][h] * w[e][n][h] over h in double and rounds once to the activation type; the kernel
adds the same exact products in fp32 (matrix cores) in another order and rounds once.  Any order of H fp32
additions of exact products is within H * 2^-24 * sum|x*w| of the true sum; the rounding to bf16 can then fall
on the other side of a rounding boundary, one bf16 ulp (2^-7 relative at most).  With small-integer inputs every
partial sum is an integer below 2^24, both sides hold the exact sum before the one rounding, and the results
must agree bit for bit: that case pins every index of the kernel (row ranges, tiles, tails, expert of a row).
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
    mod.binding.lib()
    return mod


def as64(a, dtype):
    return (a if dtype == FP32 else workloads.bf16_bits_to_f32(a)).astype(np.float64)


def to_act(a, dtype):
    return np.ascontiguousarray(a, np.float32) if dtype == FP32 else workloads.f32_to_bf16_bits(a)


def run_path(m, w, logits, x):
    """Route + dispatch + regather on the GPU; returns the buffers and the oracle's view of the same inputs."""
    import torch
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm,
                     w.padded)
    b = m.alloc_buffers(cfg, logits, x, canary=0xA5)
    m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
    torch.cuda.synchronize()
    ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor, renorm=w.renorm,
                         padded=w.padded)
    return cfg, b, ref


def expert_gpu(m, cfg, b, we, n_out, slices=(-1,), canary=0x5A):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    wd = bufs.to_device_act(cfg, we.reshape(-1, we.shape[-1]))
    L = m.monta_ws_layout_query(cfg)
    y = torch.empty((L.max_rows + 1, n_out), dtype=b.final.dtype, device="cuda:0")     # one row of canary behind the buffer
    y.view(torch.uint8).fill_(canary)
    for j in slices:
        m.monta_expert_linear(cfg, b.final, wd, n_out, y[:L.max_rows], b.ws, j)
    torch.cuda.synchronize()
    host = bufs.to_host_act(cfg, y)
    assert np.all(host[L.max_rows].view(np.uint8) == canary), "monta_expert_linear wrote past the end of y"
    return host[:L.max_rows], wd


def check_untouched(y, pl, canary=0x5A):
    """Rows of no expert's kept range keep the canary."""
    mask = np.ones(y.shape[0], bool)
    for e in range(pl.kept.shape[0]):
        mask[int(pl.offsets[e]):int(pl.offsets[e] + pl.kept[e])] = False
    assert np.all(y[mask].view(np.uint8) == canary)
    return np.nonzero(~mask)[0]


# tokens, hidden, experts, k, ep, tp, S, cf, out features, padded: ragged row tiles, two column tiles with a ragged
# second one, hidden sizes that are not whole 64-element steps (and one shorter than a step), drops, an expert
# layout with padding rows
CASES = [
    (300, 200, 6, 2, 3, 2, 2, 0.7, 264, 0),
    (1000, 64, 4, 2, 2, 1, 4, 0.0, 512, 0),
    (256, 24, 8, 1, 2, 2, 2, 0.0, 40, 0),
    (640, 136, 5, 3, 1, 2, 2, 0.5, 256, 1),
    (2048, 256, 2, 1, 2, 4, 2, 0.0, 8, 0),
    # long segments and whole 64-element steps: the direct-to-LDS kernel (256-row tiles), ragged segment ends, drops,
    # a ragged second column tile, the padded layout
    (4096, 128, 3, 2, 3, 2, 2, 0.9, 264, 0),
    (3072, 192, 2, 2, 1, 1, 3, 0.7, 512, 1),
    # more than 64 experts (the tile lookup takes two rounds of 64), with both kernels
    (2000, 72, 100, 2, 4, 1, 2, 0.0, 40, 0),
    (10240, 64, 80, 2, 4, 2, 2, 0.0, 256, 0),
    # many ragged tiles (experts x column tiles above one round of workgroups): they stay inside their segments' panels
    (10240, 64, 80, 2, 4, 2, 2, 0.0, 1024, 0),
]


@pytest.mark.parametrize("dtype", [BF16, FP32])
@pytest.mark.parametrize("case", CASES)
def test_expert_small_integers_bit_exact(m, case, dtype):
    T, H, E, k, ep, tp, S, cf, N, padded = case
    _say(f"expert ints {case} dtype={dtype}")
    w = Workload("ex", T, H, dtype, E, k, ep, tp, S, cf, padded=padded)
    logits = workloads.make_logits(w, seed=T + H)
    rng = np.random.default_rng(H + N)
    x = to_act(rng.integers(-4, 5, size=(T, H)).astype(np.float32), dtype)
    we = to_act(rng.integers(-4, 5, size=(E, N, H)).astype(np.float32), dtype)
    cfg, b, ref = run_path(m, w, logits, x)
    pl = ref.plan
    lo, hi = oracle.expert_ranges(pl, tp, S)
    want = oracle.expert(ref.final, we, lo, hi)
    got, _ = expert_gpu(m, cfg, b, we, N)
    rows = check_untouched(got, pl)
    np.testing.assert_array_equal(got[rows], want[rows])
    # slice by slice, in any order, fills the same buffer
    got2, _ = expert_gpu(m, cfg, b, we, N, slices=tuple(reversed(range(S))))
    check_untouched(got2, pl)
    np.testing.assert_array_equal(got2[rows], want[rows])
    # one slice alone writes that slice's rows and nothing else
    lj, hj = oracle.expert_ranges(pl, tp, S, 0)
    got3, _ = expert_gpu(m, cfg, b, we, N, slices=(0,))
    only = np.zeros(got3.shape[0], bool)
    for e in range(E):
        only[lj[e]:hj[e]] = True
    np.testing.assert_array_equal(got3[np.nonzero(only)[0]], want[np.nonzero(only)[0]])
    assert np.all(got3[~only].view(np.uint8) == 0x5A)


@pytest.mark.parametrize("dtype", [BF16, FP32])
@pytest.mark.parametrize("case", CASES[:4] + CASES[5:])
def test_expert_normal_inputs_within_bound(m, case, dtype):
    T, H, E, k, ep, tp, S, cf, N, padded = case
    _say(f"expert normal {case} dtype={dtype}")
    w = Workload("ex", T, H, dtype, E, k, ep, tp, S, cf, padded=padded)
    logits, x = workloads.make_inputs(w, seed=7)
    we = workloads.make_expert_weights(w, n_out=N, seed=7)
    cfg, b, ref = run_path(m, w, logits, x)
    pl = ref.plan
    lo, hi = oracle.expert_ranges(pl, tp, S)
    want = oracle.expert(ref.final, we, lo, hi)
    got, wd = expert_gpu(m, cfg, b, we, N)
    rows = check_untouched(got, pl)
    for e in range(E):
        seg = slice(int(pl.offsets[e]), int(pl.offsets[e] + pl.kept[e]))
        mag = np.abs(as64(ref.final[seg], dtype)) @ np.abs(as64(we[e], dtype)).T
        ref64 = as64(want[seg], dtype)
        tol = H * 2.0 ** -24 * mag + (2.0 ** -24 if dtype == FP32 else 2.0 ** -7) * np.abs(ref64) + 1e-30
        err = np.abs(as64(got[seg], dtype) - ref64)
        assert np.all(err <= tol), f"expert {e}: max err/tol {np.max(err / tol):.3g}"
    # repeatable bit for bit
    again, _ = expert_gpu(m, cfg, b, we, N)
    np.testing.assert_array_equal(again, got)


def test_expert_random_shapes_bit_exact(m):
    """Seeded random shapes on both kernels (long segments with whole 64-element steps, and everything else), small
    integers so that the comparison is exact; whole buffer and slice by slice."""
    rng = np.random.default_rng(2024)
    for it in range(12):
        E = int(rng.choice([1, 2, 3, 4, 6, 8]))
        k = int(rng.integers(1, min(E, 3) + 1))
        tp = int(rng.choice([1, 2, 4]))
        S = int(rng.choice([1, 2, 3, 4]))
        long_segments = it % 2 == 0
        T = S * tp * int(rng.integers(40, 90) if not long_segments else rng.integers(150, 400) * max(1, E // 2))
        H = int(rng.choice([64, 128, 192, 320]) if long_segments else rng.choice([8, 24, 72, 200, 256]))
        N = int(rng.choice([8, 64, 136, 256, 264, 520]))
        cf = float(rng.choice([0.0, 0.6, 1.1]))
        padded = int(rng.integers(0, 2))
        ep = int(rng.choice([d for d in (1, 2, 3, 4) if E % d == 0]))
        case = (T, H, E, k, ep, tp, S, cf, N, padded)
        _say(f"expert random {it}: {case}")
        w = Workload("exr", T, H, BF16, E, k, ep, tp, S, cf, padded=padded)
        logits = workloads.make_logits(w, seed=100 + it)
        x = to_act(rng.integers(-4, 5, size=(T, H)).astype(np.float32), BF16)
        we = to_act(rng.integers(-4, 5, size=(E, N, H)).astype(np.float32), BF16)
        cfg, b, ref = run_path(m, w, logits, x)
        pl = ref.plan
        lo, hi = oracle.expert_ranges(pl, tp, S)
        want = oracle.expert(ref.final, we, lo, hi)
        got, _ = expert_gpu(m, cfg, b, we, N)
        rows = check_untouched(got, pl)
        np.testing.assert_array_equal(got[rows], want[rows], err_msg=str(case))
        got2, _ = expert_gpu(m, cfg, b, we, N, slices=tuple(range(S)))
        check_untouched(got2, pl)
        np.testing.assert_array_equal(got2[rows], want[rows], err_msg=str(case))


@pytest.mark.parametrize("H", [64, 128, 320])
def test_expert_short_and_long_ragged_tiles(m, H):
    """Segment sizes fixed by the logits (top-1, one expert per token run): 2 whole tiles + 7 rows, 1 whole tile + 64
    rows (the longest "short" ragged tile), 2 whole tiles + 249 rows, and 33 rows alone.  Hidden sizes of one, two and
    five 64-element steps take the short-tile loop through its start-up, its last steps and a full turn of its three
    stages.  Small integers: exact."""
    sizes = [2 * 256 + 7, 256 + 64, 2 * 256 + 249, 33]
    T, E, N = sum(sizes), 4, 264
    _say(f"expert ragged tiles H={H} sizes={sizes}")
    w = Workload("ex-ragged", T, H, BF16, E, 1, 2, 1, 1, 0.0)
    logits = np.full((T, E), -4.0, np.float32)
    t0 = 0
    for e, n in enumerate(sizes):
        logits[t0:t0 + n, e] = 4.0
        t0 += n
    rng = np.random.default_rng(H)
    logits += rng.uniform(-0.25, 0.25, size=logits.shape).astype(np.float32)
    x = to_act(rng.integers(-4, 5, size=(T, H)).astype(np.float32), BF16)
    we = to_act(rng.integers(-4, 5, size=(E, N, H)).astype(np.float32), BF16)
    cfg, b, ref = run_path(m, w, logits, x)
    pl = ref.plan
    assert [int(v) for v in pl.kept] == sizes
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    want = oracle.expert(ref.final, we, lo, hi)
    got, _ = expert_gpu(m, cfg, b, we, N)
    rows = check_untouched(got, pl)
    np.testing.assert_array_equal(got[rows], want[rows])


def test_expert_identity_weights_reproduce_the_identity_expert_path(m):
    """w[e] = I: y equals FINAL on the kept rows, and combine of y equals combine of FINAL."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w = Workload("ex-id", 1024, 256, BF16, 8, 2, 4, 2, 2, 1.0)
    logits, x = workloads.make_inputs(w, seed=3)
    eye = workloads.f32_to_bf16_bits(np.stack([np.eye(w.hidden, dtype=np.float32)] * w.experts))
    cfg, b, ref = run_path(m, w, logits, x)
    got, _ = expert_gpu(m, cfg, b, eye, w.hidden)
    R = ref.plan.R
    np.testing.assert_array_equal(got[:R], ref.final[:R])
    y = bufs.to_device_act(cfg, got)
    m.monta_combine(cfg, y, b.gates, b.out, b.ws)
    torch.cuda.synchronize()
    same = np.all(b.gates.cpu().numpy() == ref.gates, axis=1)
    np.testing.assert_array_equal(bufs.to_host_act(cfg, b.out)[same], ref.out[same])


def test_expert_skips_an_expert_nobody_chose(m):
    w = Workload("ex-empty", 512, 128, BF16, 4, 1, 2, 2, 2, 0.0)
    logits, x = workloads.make_inputs(w, seed=5)
    logits[:, 2] = -50.0                                  # expert 2 is never chosen
    we = workloads.make_expert_weights(w, n_out=64, seed=5)
    cfg, b, ref = run_path(m, w, logits, x)
    pl = ref.plan
    assert pl.kept[2] == 0
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    want = oracle.expert(ref.final, we, lo, hi)
    got, _ = expert_gpu(m, cfg, b, we, 64)
    rows = check_untouched(got, pl)
    err = np.abs(as64(got[rows], BF16) - as64(want[rows], BF16))
    assert np.all(err <= 2.0 ** -6 * np.abs(as64(want[rows], BF16)) + 1e-6)


@pytest.mark.parametrize("case", [CASES[0], CASES[1], CASES[3], CASES[5], CASES[6]])
def test_overlapped_pipeline_gives_the_same_buffers(m, case):
    """route + slice pipeline + expert layer in one call: with and without the per-slice overlap on the side stream,
    STAGE, FINAL and y are the same as from the separate calls, run twice in a row on the same buffers."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    T, H, E, k, ep, tp, S, cf, N, padded = case
    _say(f"expert pipeline {case}")
    w = Workload("ex", T, H, BF16, E, k, ep, tp, S, cf, padded=padded)
    logits, x = workloads.make_inputs(w, seed=13)
    we = workloads.make_expert_weights(w, n_out=N, seed=13)
    cfg, b, ref = run_path(m, w, logits, x)
    want, wd = expert_gpu(m, cfg, b, we, N)
    R = ref.plan.R
    L = m.monta_ws_layout_query(cfg)
    for overlap in (0, 1, 1):
        b2 = m.alloc_buffers(cfg, logits, x, canary=0xA5)
        y = torch.empty((L.max_rows, N), dtype=b2.final.dtype, device="cuda:0")
        y.view(torch.uint8).fill_(0x5A)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for _ in range(2):
                m.monta_route_dispatch_expert(cfg, b2.logits, b2.x, b2.topk_idx, b2.gates, b2.stage, b2.final, wd, N, y,
                                              b2.ws, overlap, stream)
            m.monta_combine(cfg, b2.final, b2.gates, b2.out, b2.ws, stream)     # ordered behind the expert launches
        torch.cuda.synchronize()
        np.testing.assert_array_equal(b2.topk_idx.cpu().numpy(), ref.topk_idx)
        np.testing.assert_array_equal(bufs.to_host_act(cfg, b2.stage)[:R], ref.stage[:R])
        np.testing.assert_array_equal(bufs.to_host_act(cfg, b2.final), bufs.to_host_act(cfg, b.final))
        np.testing.assert_array_equal(bufs.to_host_act(cfg, y), want)


@pytest.mark.parametrize("overlap", [0, 1])
def test_gate_expert_step_in_a_hip_graph(m, overlap):
    """gate -> route/dispatch/expert (with and without the second stream) -> combine, captured in a HIP graph and replayed
    on changing inputs with eager work and synchronisations in between: every replay gives the eager bits."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w = Workload("ex-graph", 2048, 512, BF16, 8, 2, 4, 2, 4, 0.8)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor)
    xs = [workloads.make_inputs(w, seed=s)[1] for s in (1, 2, 3)]
    b = m.alloc_buffers(cfg, None, xs[0], canary=0)
    wg = bufs.to_device_act(cfg, workloads.make_gate_weights(w, seed=1))
    we = bufs.to_device_act(cfg, workloads.make_expert_weights(w, seed=1).reshape(-1, w.hidden))
    y = torch.zeros_like(b.final)
    stream = torch.cuda.Stream()

    def step():
        m.monta_gate(cfg, b.x, wg, b.logits, stream)
        m.monta_route_dispatch_expert(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, we, w.hidden, y, b.ws,
                                      overlap, stream)
        m.monta_combine(cfg, y, b.gates, b.out, b.ws, stream)

    def load(i):
        b.x.copy_(torch.from_numpy(xs[i].view(np.int16)).cuda().view(torch.bfloat16))
        torch.cuda.synchronize()

    def snapshot():
        torch.cuda.synchronize()
        R = m.read_tables(cfg, b.ws)["R"]
        return R, b.topk_idx.cpu().numpy(), bufs.to_host_act(cfg, y, R).copy(), bufs.to_host_act(cfg, b.out).copy()

    eager = []
    for i in range(3):
        load(i)
        with torch.cuda.stream(stream):
            step()
        eager.append(snapshot())
    assert not np.array_equal(eager[0][1], eager[1][1])   # the inputs really route differently
    load(0)
    with torch.cuda.stream(stream):
        step()                                           # side stream and events exist before the capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
    for rep in range(2):
        for i in (2, 0, 1):
            _say(f"expert graph overlap={overlap} rep={rep} input={i}")
            load(i)
            b.out.zero_()
            y.zero_()
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot()
            assert got[0] == eager[i][0]
            for a_, b_ in zip(got[1:], eager[i][1:]):
                np.testing.assert_array_equal(a_, b_)


@pytest.mark.parametrize("name", ["mixtral", "2x70b"])
def test_expert_named_workloads_full_size(m, name):
    """Full-size launch (N = H); the oracle recomputes a sample of rows, among them each segment's first and last."""
    w = workloads.CONFIGS[name]
    _say(f"expert workload {name}")
    logits, x = workloads.make_inputs(w)
    we = workloads.make_expert_weights(w)
    cfg, b, ref = run_path(m, w, logits, x)
    pl = ref.plan
    got, _ = expert_gpu(m, cfg, b, we, w.hidden)
    check_untouched(got, pl)
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    rng = np.random.default_rng(9)
    rows = [int(r) for e in range(w.experts) if hi[e] > lo[e] for r in (lo[e], hi[e] - 1)]
    rows += [int(r) for r in rng.integers(0, pl.R, size=max(4, 24 - len(rows)))]
    rows = np.unique(np.array(rows, np.int32))
    want = oracle.expert(ref.final, we, lo, hi, only_rows=rows)
    expert_of = np.searchsorted(np.asarray(pl.offsets[1:w.experts + 1]), rows, side="right")
    for r, e in zip(rows, expert_of):
        mag = np.abs(as64(ref.final[r], BF16)) @ np.abs(as64(we[e], BF16)).T
        ref64 = as64(want[r], BF16)
        tol = w.hidden * 2.0 ** -24 * mag + 2.0 ** -7 * np.abs(ref64) + 1e-30
        err = np.abs(as64(got[r], BF16) - ref64)
        assert np.all(err <= tol), f"row {r} expert {e}: max err/tol {np.max(err / tol):.3g}"
        # the typical error is rounding to bf16 only: a dropped or doubled step of the hidden axis is not
        assert np.sqrt(np.mean(err ** 2)) <= 2.0 ** -8 * np.sqrt(np.mean(ref64 ** 2))
