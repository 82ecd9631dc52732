"""The entry point that allocates nothing (plan tables in the library's static device array) against the
existing calls it is a variant of: monta_route_dispatch_regather + monta_combine with a caller workspace.
Same kernels, so every output must be bit-identical.  Two calls in a row share the array; the second is a
smaller problem of another shape, so stale tables of the first must not leak into it."""
import sys

import numpy as np
import pytest

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


def _both_ways(m, w, seed):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    logits, x = workloads.make_inputs(w, seed=seed)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm,
                     w.padded)
    ref = m.alloc_buffers(cfg, logits, x, canary=0xA5)
    m.monta_route_dispatch_regather(cfg, ref.logits, ref.x, ref.topk_idx, ref.gates, ref.stage, ref.final, ref.ws)
    m.monta_combine(cfg, ref.final, ref.gates, ref.out, ref.ws)
    torch.cuda.synchronize()
    got = m.alloc_buffers(cfg, logits, x, canary=0xA5)          # its workspace stays unused
    got.topk_idx.fill_(-7)
    got.gates.fill_(-7.0)
    m.monta_route_dispatch_combine_static(cfg, got.logits, got.x, got.topk_idx, got.gates, got.stage, got.final, got.out)
    torch.cuda.synchronize()
    R = m.read_tables(cfg, ref.ws)["R"]
    assert R > 0
    assert torch.equal(got.topk_idx, ref.topk_idx)
    assert torch.equal(got.gates.view(torch.int32), ref.gates.view(torch.int32))
    for name in ("stage", "final", "out"):
        a = bufs.to_host_act(cfg, getattr(got, name))
        b = bufs.to_host_act(cfg, getattr(ref, name))
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), name      # canary rows above R included
    return R


def test_static_scratch_call_matches_the_workspace_calls_twice_in_a_row(m):
    big = Workload("noalloc-big", 6144, 1536, BF16, 16, 4, 4, 2, 4, 0.8, zipf_s=0.9)
    small = Workload("noalloc-small", 768, 264, FP32, 6, 2, 3, 2, 2, 0.0)
    for mode in (-1, 1, 2, 0):          # 0 is replaced by the size-chosen mode inside the call
        m.monta_set_pipeline_mode(mode)
        for w, seed in ((big, 1), (small, 2), (big, 3)):
            _say(f"static scratch: {w.name} seed={seed} mode={mode}")
            _both_ways(m, w, seed)
    m.monta_set_pipeline_mode(-1)


def test_static_scratch_call_on_a_named_workload_and_with_profiling_on(m):
    w = workloads.CONFIGS["mixtral"]
    _say("static scratch: mixtral")
    _both_ways(m, w, 0)
    _say("static scratch: tiny right after (smaller, other shape)")
    _both_ways(m, workloads.CONFIGS["tiny"], 0)
    # with event profiling on the call is refused: it must not create events
    import torch
    cfg = m.make_cfg(256, 128, FP32, 4, 2, 2, 2, 2, 0.0)
    b = m.alloc_buffers(cfg, *workloads.make_inputs(workloads.CONFIGS["tiny"]))
    m.monta_profile_enable(True)
    try:
        with pytest.raises(m.MontaError):
            m.monta_route_dispatch_combine_static(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.out)
    finally:
        m.monta_profile_enable(False)
        m.monta_profile_reset()
    torch.cuda.synchronize()


def test_static_scratch_call_replayed_from_a_hip_graph(m):
    """The callers it is for: captured once (after one eager call, which looks the array's address up), replayed
    on changing inputs with eager work in between; every replay must give the eager bits."""
    import torch
    w = Workload("noalloc-graph", 4096, 1024, BF16, 8, 2, 4, 2, 4, 0.8, zipf_s=0.6)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm)
    inputs = [workloads.make_inputs(w, seed=s) for s in (1, 2, 3)]
    b = m.alloc_buffers(cfg, *inputs[0], canary=0)
    stream = torch.cuda.Stream()

    def step():
        m.monta_route_dispatch_combine_static(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.out, stream)

    def load(i):
        logits, x = inputs[i]
        b.logits.copy_(torch.from_numpy(logits).cuda())
        b.x.copy_(torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16))
        torch.cuda.synchronize()

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (b.topk_idx, b.gates.view(torch.int32), b.out.view(torch.int16))]

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
            _say(f"static scratch: graph replay rep={rep} input={i}")
            load(i)
            b.out.zero_()
            b.topk_idx.zero_()
            graph.replay()
            got = snapshot()
            for a_, e_ in zip(got, eager[i]):
                assert torch.equal(a_, e_)
            # eager work of the same library between replays (it uses its own workspace, not the static array)
            b2 = m.alloc_buffers(cfg, *inputs[(i + 1) % 3])
            m.monta_route_dispatch_regather(cfg, b2.logits, b2.x, b2.topk_idx, b2.gates, b2.stage, b2.final, b2.ws)
            torch.cuda.synchronize()
            del b2
