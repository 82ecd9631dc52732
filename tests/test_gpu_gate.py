"""GPU parity of the gate projection (monta_gate) against the CPU oracle.

Bar.  The oracle sums x[t][h] * w[e][h] over h in double and rounds once to fp32; the
kernel adds the same exact products in fp32 in another order.  For any order of n
fp32 additions of exact products the result differs from the true sum by at most
(n - 1) * 2^-24 * sum |x*w| (first order), so the tolerance per logit is
H * 2^-24 * sum_h |x[t][h] * w[e][h]| plus half an fp32 ulp of the oracle's own
rounding.  With small-integer inputs every partial sum is an integer below 2^24,
every order gives the same fp32 value, and the two sides must agree bit for bit:
that case pins every index of the kernel (rows, hidden pieces, expert tiles, tails).
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


def gate_gpu(m, T, H, E, dtype, x, wg, canary=True):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    cfg = m.make_cfg(T, H, dtype, E, 1, 1, 1, 1, 0.0)
    xd = bufs.to_device_act(cfg, x)
    wd = bufs.to_device_act(cfg, wg)
    # one row of canary behind the logits: the kernel must not write past [T][E]
    out = torch.full((T + 1, E), float("nan"), dtype=torch.float32, device="cuda:0")
    m.monta_gate(cfg, xd, wd, out[:T])
    torch.cuda.synchronize()
    host = out.cpu().numpy()
    assert np.all(np.isnan(host[T])), "monta_gate wrote past the end of logits"
    return host[:T].copy(), (cfg, xd, wd)


def as_f64(a, dtype):
    return (a if dtype == FP32 else workloads.bf16_bits_to_f32(a)).astype(np.float64)


def to_act(a, dtype):
    return np.ascontiguousarray(a, np.float32) if dtype == FP32 else workloads.f32_to_bf16_bits(a)


# (T, H, E): several 32-token tiles with a ragged last one, hidden sizes that are not whole 64-element blocks,
# expert counts on both sides of the 32-wide tiles up to the library's limit
SHAPES = [(1, 8, 1), (31, 64, 7), (100, 200, 8), (257, 1032, 33), (64, 4096, 64), (96, 72, 100), (40, 520, 256),
          (1000, 4096, 8), (33, 8, 129),
          # at most 8 experts and whole 64-element quarters: the persistent whole-row kernel, one and two chunks per row,
          # quarters that are not powers of two, fewer MFMA steps than waves, more groups than workgroups
          (70, 8192, 8), (45, 7168, 3), (19, 1088, 5), (300, 2048, 2), (64, 128, 8), (9, 4160, 1), (5000, 256, 6),
          # whole chunks of 512 / 1024 / 2048 elements: the direct-to-LDS form (one to seven chunks a row, ragged last group,
          # more groups than workgroups)
          (50, 1024, 3), (77, 512, 8), (130, 1536, 5), (3000, 2048, 8), (9, 6144, 2), (300, 5120, 7), (4100, 512, 4),
          # many tokens and more than 32 experts: 128-token workgroups, a wave per output tile (one, two and four
          # tiles per wave), ragged last workgroup, hidden sizes that are not whole steps
          (32773, 64, 64), (32800, 72, 100), (32769, 136, 200), (33000, 200, 33)]


@pytest.mark.parametrize("dtype", [BF16, FP32])
@pytest.mark.parametrize("T,H,E", SHAPES)
def test_gate_small_integers_bit_exact(m, T, H, E, dtype):
    _say(f"gate ints T={T} H={H} E={E} dtype={dtype}")
    rng = np.random.default_rng(T * 7 + H + E)
    x = to_act(rng.integers(-8, 9, size=(T, H)).astype(np.float32), dtype)
    wg = to_act(rng.integers(-8, 9, size=(E, H)).astype(np.float32), dtype)
    want = oracle.gate(x, wg)
    got, _ = gate_gpu(m, T, H, E, dtype, x, wg)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("dtype", [BF16, FP32])
@pytest.mark.parametrize("T,H,E", SHAPES)
def test_gate_normal_inputs_within_bound(m, T, H, E, dtype):
    _say(f"gate normal T={T} H={H} E={E} dtype={dtype}")
    w = Workload("g", T, H, dtype, E, 1, 1, 1, 1, 0.0)
    _, x = workloads.make_inputs(w, seed=3)
    wg = workloads.make_gate_weights(w, seed=3)
    want = oracle.gate(x, wg).astype(np.float64)
    got, (cfg, xd, wd) = gate_gpu(m, T, H, E, dtype, x, wg)
    mag = np.abs(as_f64(x, dtype)) @ np.abs(as_f64(wg, dtype)).T
    tol = H * 2.0 ** -24 * mag + 2.0 ** -24 * np.abs(want) + 1e-30
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= tol), f"max err/tol {np.max(err / tol):.3g}"
    # same inputs, same shape: the order of the additions is fixed, so a second call agrees bit for bit
    import torch
    again = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    m.monta_gate(cfg, xd, wd, again)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(again.cpu().numpy(), got)


@pytest.mark.parametrize("name", ["tiny", "mixtral", "2x70b", "longctx", "skewed"])
def test_gate_named_workloads_full_size(m, name):
    """Full-size launch; the oracle recomputes a sample of token rows (all of them where that takes seconds)."""
    w = workloads.CONFIGS[name]
    _say(f"gate workload {name}")
    _, x = workloads.make_inputs(w)
    wg = workloads.make_gate_weights(w)
    got, _ = gate_gpu(m, w.tokens, w.hidden, w.experts, w.dtype, x, wg)
    budget = 4e8                                        # multiply-adds the oracle is asked for
    n = int(min(w.tokens, max(64, budget // (w.hidden * w.experts))))
    rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(w.tokens - 40, w.tokens),
                                     np.random.default_rng(5).integers(0, w.tokens, size=n)]))
    rows = rows[(rows >= 0) & (rows < w.tokens)]
    want = oracle.gate(x[rows], wg).astype(np.float64)
    mag = np.abs(as_f64(x[rows], w.dtype)) @ np.abs(as_f64(wg, w.dtype)).T
    tol = w.hidden * 2.0 ** -24 * mag + 2.0 ** -24 * np.abs(want)
    err = np.abs(got[rows].astype(np.float64) - want)
    assert np.all(err <= tol), f"max err/tol {np.max(err / tol):.3g}"
    # the typical error of an fp32 sum is far below the worst-case bound; a dropped or doubled piece of the
    # hidden axis is not
    assert np.sqrt(np.mean(err ** 2)) <= 2.0 ** -16 * np.sqrt(np.mean(want ** 2)) + 1e-12
    assert np.all(np.isfinite(got))


def test_gate_feeds_the_routing_path(m):
    """Gate -> route/dispatch/regather -> combine on the GPU against the oracle run from its OWN logits.

    A GPU logit may differ from the oracle's within the projection's tolerance, which can flip a choice only where two
    logits of a token are closer than that.  So: tokens whose top-(k+1) logits are further apart than the tolerance
    ("decided", all but a few) must get the oracle's experts in the oracle's order; for the others the chosen experts
    must be within tolerance of the oracle's k-th logit; and when no choice flipped (the expected outcome: the
    worst-case tolerance is far above the error of a real fp32 sum) every table and buffer must match."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w = Workload("g2r", 1024, 512, BF16, 16, 2, 4, 2, 2, 1.0)
    k = w.top_k
    _, x = workloads.make_inputs(w, seed=11)
    wg = workloads.make_gate_weights(w, seed=11)
    logits = oracle.gate(x, wg)
    ref = oracle.forward(logits, x, k=k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    R = ref.plan.R
    assert 0 < R < w.tokens * k                  # the case has drops

    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, k, w.ep, w.tp, w.slices, w.capacity_factor)
    b = m.alloc_buffers(cfg, None, x, canary=0xA5)
    wd = bufs.to_device_act(cfg, wg)
    m.monta_gate(cfg, b.x, wd, b.logits)
    m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
    m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
    torch.cuda.synchronize()
    got_idx = b.topk_idx.cpu().numpy()

    l64 = logits.astype(np.float64)
    tol = w.hidden * 2.0 ** -24 * (np.abs(as_f64(x, BF16)) @ np.abs(as_f64(wg, BF16)).T) + 2.0 ** -24 * np.abs(l64)
    order = np.argsort(-l64, axis=1, kind="stable")
    srt = np.take_along_axis(l64, order, axis=1)
    tsrt = np.take_along_axis(tol, order, axis=1)
    gaps = srt[:, :k] - srt[:, 1:k + 1]                                  # between ranks j and j+1, j < k
    decided = np.all(gaps > tsrt[:, :k] + tsrt[:, 1:k + 1], axis=1)
    assert decided.mean() > 0.95
    np.testing.assert_array_equal(got_idx[decided], ref.topk_idx[decided])
    # undecided tokens: every chosen expert is within tolerance of the oracle's k-th largest logit
    rows = np.nonzero(~decided)[0]
    for t in rows:
        kth = srt[t, k - 1]
        for e in got_idx[t]:
            assert l64[t, e] >= kth - (tol[t, e] + tsrt[t, k - 1]), (t, e)
        assert len(set(got_idx[t].tolist())) == k

    if np.array_equal(got_idx, ref.topk_idx):
        tabs = m.read_tables(cfg, b.ws)
        assert tabs["R"] == R
        np.testing.assert_array_equal(tabs["pos_final"], ref.plan.pos_final)
        np.testing.assert_array_equal(bufs.to_host_act(cfg, b.final)[:R], ref.final[:R])
        # gates come from logits that differ within tol: softmax moves by at most the largest logit difference
        gd = np.abs(b.gates.cpu().numpy().astype(np.float64) - ref.gates.astype(np.float64))
        assert np.all(gd <= 2.0 * tol.max(axis=1, keepdims=True) + 1e-6)
        d = np.abs(workloads.bf16_bits_to_f32(bufs.to_host_act(cfg, b.out)).astype(np.float64)
                   - workloads.bf16_bits_to_f32(ref.out).astype(np.float64))
        assert d.max() <= 1e-2                   # the bf16 bar of the combine step
    else:
        _say("a near-tie flipped between the two gate projections: buffers not compared")
