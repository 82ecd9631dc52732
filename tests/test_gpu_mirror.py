"""GPU parity of the mirrored return path (monta_unregather, monta_combine_staged,
monta_unregather_combine) against the oracle: bit-exact row movement, and a combine result that
is bitwise the direct monta_combine result (same sum in the same order)."""
import sys

import numpy as np
import pytest

import oracle
import workloads
from workloads import BF16, FP32, Workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def m():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_00662_amd as mod
    mod.binding.lib()
    return mod


CASES = [
    workloads.CONFIGS["tiny"],
    Workload("m1", 330, 40, BF16, 5, 3, 5, 2, 3, 0.7, zipf_s=0.8),
    Workload("m2", 4096, 1028, FP32, 16, 4, 4, 2, 2, 0.3, zipf_s=0.8),
    Workload("m3", 2048, 7168, BF16, 32, 8, 8, 4, 4, 0.25, zipf_s=0.8),
    Workload("m4", 777, 100, FP32, 256, 32, 16, 7, 3, 0.9, zipf_s=0.8),
    workloads.CONFIGS["mixtral"],
    workloads.CONFIGS["2x70b"],
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_mirrored_return_path(m, w):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    print(f"mirror {w.name}", flush=True)
    sys.stdout.flush()
    logits, x = workloads.make_inputs(w, seed=w.tokens % 7)
    ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
    R = ref.plan.R
    rng = np.random.default_rng(3)
    y = rng.standard_normal((R, w.hidden), dtype=np.float32) * 2
    if w.dtype == BF16:
        y = workloads.f32_to_bf16_bits(y)
    ys_ref = oracle.unregather(y, ref.plan, w.tp, w.slices)
    out_ref = oracle.combine(y, ref.gates, ref.plan.pos_final)

    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm)
    b = m.alloc_buffers(cfg, logits, x, canary=0xA5)
    m.monta_set_pipeline_mode(1)
    m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
    b.gates.copy_(torch.from_numpy(ref.gates).cuda())        # both sides combine with the same gates
    ydev = torch.empty_like(b.final)
    ydev.view(torch.uint8).fill_(0x5A)
    ydev[:R].copy_(bufs.to_device_act(cfg, y))

    def fresh():
        ys = torch.empty_like(b.final)
        ys.view(torch.uint8).fill_(0xA5)
        out = torch.empty_like(b.out)
        out.view(torch.uint8).fill_(0xA5)
        return ys, out

    def check(ys, out, what):
        torch.cuda.synchronize()
        ys_h = bufs.to_host_act(cfg, ys)
        np.testing.assert_array_equal(ys_h[:R], ys_ref, err_msg=f"{what}: y_stage")
        assert (ys_h[R:].view(np.uint8) == 0xA5).all(), f"{what}: rows past R were written"
        np.testing.assert_array_equal(bufs.to_host_act(cfg, out), out_ref, err_msg=f"{what}: out")

    # whole-buffer calls
    ys, out = fresh()
    m.monta_unregather(cfg, ydev, ys, b.ws, -1)
    m.monta_combine_staged(cfg, ys, b.gates, out, b.ws, -1)
    check(ys, out, "all")
    # slice by slice, unregather in reverse order, then combine in forward order
    ys, out = fresh()
    for j in reversed(range(w.slices)):
        m.monta_unregather(cfg, ydev, ys, b.ws, j)
    for j in range(w.slices):
        m.monta_combine_staged(cfg, ys, b.gates, out, b.ws, j)
    check(ys, out, "slices")
    # the pipeline, twice in a row on the same buffers
    ys, out = fresh()
    for _ in range(2):
        m.monta_unregather_combine(cfg, ydev, ys, b.gates, out, b.ws)
    check(ys, out, "pipeline")
    # the direct combine of the same y gives the same bits
    out2 = torch.empty_like(b.out)
    m.monta_combine(cfg, ydev, b.gates, out2, b.ws)
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.uint8), out.view(torch.uint8))


def test_identity_experts_return_the_send_buffer(m):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w = Workload("m5", 1024, 512, BF16, 8, 2, 4, 2, 4, 0.8, zipf_s=1.0)
    logits, x = workloads.make_inputs(w, seed=1)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm)
    b = m.alloc_buffers(cfg, logits, x, canary=0)
    m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
    ys = torch.zeros_like(b.stage)
    m.monta_unregather(cfg, b.final, ys, b.ws, -1)
    torch.cuda.synchronize()
    R = m.read_tables(cfg, b.ws)["R"]
    assert 0 < R < w.tokens * w.top_k
    assert torch.equal(ys[:R].view(torch.int16), b.stage[:R].view(torch.int16))


def test_two_pass_gather_then_copy(m):
    """monta_allgather + monta_regather from the gathered buffer equals the fused regather, slice by slice."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    for w in (Workload("g1", 1320, 264, BF16, 6, 3, 3, 5, 4, 0.7, zipf_s=0.8), workloads.CONFIGS["mixtral"]):
        print(f"two-pass {w.name}", flush=True)
        logits, x = workloads.make_inputs(w, seed=4)
        ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor)
        R = ref.plan.R
        cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm)
        b = m.alloc_buffers(cfg, logits, x, canary=0xA5)
        gathered = torch.empty_like(b.stage)
        gathered.view(torch.uint8).fill_(0xA5)
        m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
        m.monta_dispatch(cfg, b.x, b.stage, b.ws, -1)
        for j in reversed(range(w.slices)):
            m.monta_allgather(cfg, b.stage, gathered, b.ws, j)
            m.monta_regather(cfg, gathered, b.final, b.ws, j)
        torch.cuda.synchronize()
        gh = bufs.to_host_act(cfg, gathered)
        np.testing.assert_array_equal(gh[:R], oracle.allgather(ref.stage, ref.plan, w.tp, w.slices))
        assert (gh[R:].view(np.uint8) == 0xA5).all()
        fh = bufs.to_host_act(cfg, b.final)
        np.testing.assert_array_equal(fh[:R], ref.final)
        assert (fh[R:].view(np.uint8) == 0xA5).all()
        g2 = torch.zeros_like(b.stage)
        m.monta_allgather(cfg, b.stage, g2, b.ws, -1)
        torch.cuda.synchronize()
        assert torch.equal(g2[:R].view(torch.int16 if w.dtype == BF16 else torch.int32),
                           b.stage[:R].view(torch.int16 if w.dtype == BF16 else torch.int32))


@pytest.mark.parametrize("w", [Workload("g2", 1320, 264, BF16, 6, 3, 3, 5, 4, 0.7, zipf_s=0.8),
                               Workload("g3", 900, 72, FP32, 5, 2, 5, 3, 1, 0.0),
                               Workload("g4", 2048, 512, BF16, 8, 2, 4, 2, 4, 1.25, zipf_s=0.5, padded=1),
                               workloads.CONFIGS["mixtral"], workloads.CONFIGS["2x70b"]], ids=lambda w: w.name)
def test_pipelined_two_pass_gather_and_copy(m, w):
    """The gather of chunk j+1 overlapping the D2D copy of chunk j (Fig. 8 order), in all three schedules:
    `gathered` must equal the oracle's gathered buffer and FINAL the oracle's FINAL, canaries intact."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    logits, x = workloads.make_inputs(w, seed=6)
    ref = oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor, padded=w.padded)
    R = ref.plan.R
    gathered_ref = oracle.allgather(ref.stage, ref.plan, w.tp, w.slices)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm, w.padded)
    b = m.alloc_buffers(cfg, logits, x, canary=0xA5)
    m.monta_route(cfg, b.logits, b.topk_idx, b.gates, b.ws)
    m.monta_dispatch(cfg, b.x, b.stage, b.ws, -1)
    rows_final = ref.plan.final_rows
    for schedule in (0, 1, 2, 1):
        print(f"pipelined two-pass {w.name} schedule={schedule}", flush=True)
        gathered = torch.empty_like(b.stage)
        gathered.view(torch.uint8).fill_(0xA5)
        b.final.view(torch.uint8).fill_(0xA5)
        m.monta_allgather_regather(cfg, b.stage, gathered, b.final, b.ws, schedule)
        torch.cuda.synchronize()
        gh = bufs.to_host_act(cfg, gathered)
        np.testing.assert_array_equal(gh[:R], gathered_ref)
        assert (gh[R:].view(np.uint8) == 0xA5).all()
        fh = bufs.to_host_act(cfg, b.final)
        if w.padded:
            np.testing.assert_array_equal(fh[:rows_final], ref.final)
        else:
            np.testing.assert_array_equal(fh[:R], ref.final)
        assert (fh[rows_final:].view(np.uint8) == 0xA5).all()
    with pytest.raises(m.MontaError):
        m.monta_allgather_regather(cfg, b.stage, b.stage, b.final, b.ws, 1)
    with pytest.raises(m.MontaError):
        m.monta_allgather_regather(cfg, b.stage, gathered, b.final, b.ws, 3)
