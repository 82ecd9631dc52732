"""The rows built beyond the headline path (mirrored return path, two-pass orders, capacity-padded layout, expert
layer) at the full size of the two largest workloads, `longctx` and `skewed`, against the CPU oracle.

The oracle's forward pass of a workload is computed once per module and shared.  The expert output y fed to the
return path is the oracle's FINAL with its rows rotated by one (a cheap y that differs from FINAL row by row);
both sides combine with the oracle's gates, so everything here is compared bit for bit.  The expert layer is
checked on sampled rows (first and last row of every expert's segment), within the bound of an fp32 sum in any
order plus one bf16 rounding.
"""
import sys

import numpy as np
import pytest

import oracle
import workloads
from workloads import BF16

pytestmark = pytest.mark.gpu

_REF = {}


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


def reference(name):
    if name not in _REF:
        w = workloads.CONFIGS[name]
        logits, x = workloads.make_inputs(w)
        _say(f"{name}: oracle forward")
        _REF[name] = (w, logits, x, oracle.forward(logits, x, k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor,
                                                   renorm=w.renorm))
    return _REF[name]


def gpu_path(m, w, logits, x, ref, canary=0xA5):
    """route + dispatch + regather on the GPU, then the oracle's gates put in place of the GPU's."""
    import torch
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm,
                     w.padded)
    b = m.alloc_buffers(cfg, logits, x, canary=canary)
    m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
    torch.cuda.synchronize()
    assert m.read_tables(cfg, b.ws)["R"] == ref.plan.R
    b.gates.copy_(torch.from_numpy(ref.gates).cuda())
    return cfg, b


@pytest.mark.parametrize("name", ["longctx", "skewed"])
def test_mirrored_return_path_full_size(m, name):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w, logits, x, ref = reference(name)
    R = ref.plan.R
    y = np.roll(ref.final, -1, axis=0)                  # row i of y = row i+1 of FINAL
    _say(f"{name}: oracle unregather + combine of y")
    ys_ref = oracle.unregather(y, ref.plan, w.tp, w.slices)
    out_ref = oracle.combine(y, ref.gates, ref.plan.pos_final)
    cfg, b = gpu_path(m, w, logits, x, ref)
    ydev = torch.empty_like(b.final)
    ydev.view(torch.uint8).fill_(0x5A)
    ydev[:R].copy_(bufs.to_device_act(cfg, y))
    del y
    for what in ("calls", "pipeline"):
        _say(f"{name}: mirrored return path, {what}")
        ys = torch.empty_like(b.final)
        ys.view(torch.uint8).fill_(0xA5)
        b.out.view(torch.uint8).fill_(0xA5)
        if what == "calls":
            for j in reversed(range(w.slices)):
                m.monta_unregather(cfg, ydev, ys, b.ws, j)
            m.monta_combine_staged(cfg, ys, b.gates, b.out, b.ws, -1)
        else:
            m.monta_unregather_combine(cfg, ydev, ys, b.gates, b.out, b.ws)
        torch.cuda.synchronize()
        ys_h = bufs.to_host_act(cfg, ys)
        assert np.array_equal(ys_h[:R], ys_ref), "y_stage"
        tail = ys_h[R:]
        assert (tail[:: max(1, tail.shape[0] // 2048)].view(np.uint8) == 0xA5).all() and (tail[:32].view(np.uint8) == 0xA5).all()
        del ys_h, tail, ys
        assert np.array_equal(bufs.to_host_act(cfg, b.out), out_ref), "out"
    # the direct combine of the same y: same bits
    m.monta_combine(cfg, ydev, b.gates, b.out, b.ws)
    torch.cuda.synchronize()
    assert np.array_equal(bufs.to_host_act(cfg, b.out), out_ref)


@pytest.mark.parametrize("name", ["longctx", "skewed"])
def test_two_pass_orders_full_size(m, name):
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w, logits, x, ref = reference(name)
    R = ref.plan.R
    cfg, b = gpu_path(m, w, logits, x, ref)
    gathered = torch.empty_like(b.stage)
    for schedule in (1, 2):
        _say(f"{name}: pipelined two-pass, schedule {schedule}")
        gathered.view(torch.uint8).fill_(0xA5)
        b.final.view(torch.uint8).fill_(0xA5)
        m.monta_allgather_regather(cfg, b.stage, gathered, b.final, b.ws, schedule)
        torch.cuda.synchronize()
        gh = bufs.to_host_act(cfg, gathered, R + 64)
        assert np.array_equal(gh[:R], ref.stage) and (gh[R:].view(np.uint8) == 0xA5).all()
        del gh
        fh = bufs.to_host_act(cfg, b.final, R + 64)
        assert np.array_equal(fh[:R], ref.final) and (fh[R:].view(np.uint8) == 0xA5).all()
        del fh


def test_padded_layout_skewed_full_size(m):
    """The capacity tensor [64][10240][7168] of the largest workload: kept rows, zero padding, same combine."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w0, logits, x, ref0 = reference("skewed")
    w = w0.with_(padded=1)
    _say("skewed padded: oracle plan, regather and pad")
    pl = oracle.plan(ref0.topk_idx, w.experts, w.ep, w.tp, w.slices, w.capacity_factor, padded=1)
    assert pl.final_rows == w.experts * pl.C and pl.R == ref0.plan.R
    final_ref = oracle.pad(oracle.regather(ref0.stage, pl, w.tp, w.slices, fill=0x5A5A), pl)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm, 1)
    b = m.alloc_buffers(cfg, logits, x, canary=0xA5)
    _say("skewed padded: gpu")
    m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws)
    b.gates.copy_(torch.from_numpy(ref0.gates).cuda())
    m.monta_combine(cfg, b.final, b.gates, b.out, b.ws)
    torch.cuda.synchronize()
    tabs = m.read_tables(cfg, b.ws)
    for tname in ("counts", "kept", "offsets", "pos_final", "pos_stage", "n", "stage_off", "unit_base", "send_rows"):
        assert np.array_equal(tabs[tname], getattr(pl, tname)), tname
    assert tabs["final_rows"] == pl.final_rows
    assert np.array_equal(bufs.to_host_act(cfg, b.stage, pl.R), ref0.stage)
    fh = bufs.to_host_act(cfg, b.final)
    assert fh.shape[0] == pl.final_rows
    assert np.array_equal(fh, final_ref)
    del fh, final_ref
    # the combine does not care about the layout
    assert np.array_equal(bufs.to_host_act(cfg, b.out), ref0.out)


def test_expert_layer_skewed_full_size(m):
    """64 experts, 233178 kept rows of 7168, N = H: first and last row of every segment against the oracle."""
    import torch
    from paper_2411_00662_amd import buffers as bufs
    w, logits, x, ref = reference("skewed")
    pl = ref.plan
    cfg, b = gpu_path(m, w, logits, x, ref)
    H = w.hidden
    gen = torch.Generator(device="cuda").manual_seed(77)
    wdev = torch.empty((w.experts, H, H), dtype=torch.bfloat16, device="cuda")
    for e in range(w.experts):          # drawn on the device: the host copy is only needed for the sampled rows
        wdev[e] = (torch.randn((H, H), generator=gen, device="cuda") / H ** 0.5).to(torch.bfloat16)
    L = m.monta_ws_layout_query(cfg)
    y = torch.empty((L.max_rows, H), dtype=torch.bfloat16, device="cuda")
    y.view(torch.uint8).fill_(0x5A)
    _say("skewed: expert layer on the gpu")
    m.monta_expert_linear(cfg, b.final, wdev, H, y, b.ws, -1)
    torch.cuda.synchronize()
    lo, hi = oracle.expert_ranges(pl, w.tp, w.slices)
    rows = np.unique(np.array([int(r) for e in range(w.experts) if hi[e] > lo[e] for r in (lo[e], hi[e] - 1)], np.int32))
    assert rows.size >= w.experts
    # rows past R stay untouched
    assert (bufs.to_host_act(cfg, y[pl.R:pl.R + 64]).view(np.uint8) == 0x5A).all()
    we = wdev.view(torch.int16).cpu().numpy().view(np.uint16)
    got = {int(r): bufs.to_host_act(cfg, y[int(r):int(r) + 1])[0] for r in rows}
    _say(f"skewed: oracle expert layer on {rows.size} sampled rows")
    want = oracle.expert(ref.final, we, lo, hi, only_rows=rows)

    def f64(a):
        return workloads.bf16_bits_to_f32(a).astype(np.float64)

    expert_of = np.searchsorted(np.asarray(pl.offsets[1:w.experts + 1]), rows, side="right")
    for r, e in zip(rows, expert_of):
        mag = np.abs(f64(ref.final[r])) @ np.abs(f64(we[e])).T
        ref64 = f64(want[r])
        tol = H * 2.0 ** -24 * mag + 2.0 ** -7 * np.abs(ref64) + 1e-30
        err = np.abs(f64(got[int(r)]) - ref64)
        assert np.all(err <= tol), f"row {r} expert {e}: max err/tol {np.max(err / tol):.3g}"
        assert np.sqrt(np.mean(err ** 2)) <= 2.0 ** -8 * np.sqrt(np.mean(ref64 ** 2))
