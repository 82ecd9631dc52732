#!/usr/bin/env python3
"""Benchmark of the MoE dispatch + combine hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: monta_route (top-k, gates, counting-sort plan) ->
monta_dispatch_regather (S-slice pack / regather pipeline) -> monta_combine
(identity experts: the expert output is FINAL).

The default workload is the largest one that fits one GPU (`skewed`: 65536 tokens
of 7168 bf16, 64 experts, top-8, capacity drops).  Prints ONE JSON line.  `value`
is tokens/s of the whole job on that workload; `roofline` is the dominant kernel's
algorithmic bytes per launch over its average launch duration, measured here with
HIP events on the launching stream; `cpu_baseline` is the CPU oracle timed on this
host (all cores, and one thread); `other_configs` repeats the step timing, briefly,
on the other named workloads so that one run shows all of them.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published peak


def algorithmic_bytes(w, tabs):
    """Bytes the method itself must move (per kernel class and per pipeline launch)."""
    row = w.row_bytes
    T, k, E, S, tp = w.tokens, w.top_k, w.experts, w.slices, w.tp
    pos = tabs["pos_final"]
    alive_tok = (pos >= 0).any(axis=1)
    per_slice_tok = T // S
    alive_s = alive_tok.reshape(S, per_slice_tok).sum(axis=1).astype(np.int64)
    rows_s = tabs["n"].reshape(S, tp * E).sum(axis=1).astype(np.int64)
    R = int(rows_s.sum())
    alive = int(alive_s.sum())
    idx_bytes = T * E * 4 + T * k * 8 + 6 * T * k * 4
    out = {
        "row": row, "R": R, "alive": alive,
        "route": T * E * 4 + T * k * 8, "plan": 6 * T * k * 4,
        "pack": (alive + R) * row + T * k * 4,
        "regather": 2 * R * row + R * 4,
        "combine": (R + T) * row + T * k * 8,
        "pack_s": [(int(alive_s[j]) + int(rows_s[j])) * row for j in range(S)],
        "regather_s": [2 * int(rows_s[j]) * row for j in range(S)],
    }
    out["total"] = (alive + T + 4 * R) * row + idx_bytes
    return out


def mode_label(mode):
    return "auto" if mode < 0 else str(mode)


def measure(args, w, steps, warmup, full):
    """Times `steps` steps of workload w.  full: also the per-kernel event pass and everything the headline line
    carries; otherwise only the step time and the byte accounting."""
    import torch
    import workloads
    import paper_2411_00662_amd as m

    mode = m.monta_get_pipeline_mode()
    logits, x = workloads.make_inputs(w)
    cfg = m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices, w.capacity_factor, w.renorm,
                     w.padded)
    b = m.alloc_buffers(cfg, logits, x)
    stream = torch.cuda.Stream()          # default priority; the whole step is enqueued on it

    mirror = full and args.return_path == "mirror"
    gate = full and args.gate
    experts = full and args.experts
    y_stage = torch.empty_like(b.stage) if mirror else None
    w_gate_host = workloads.make_gate_weights(w) if gate else None
    w_gate = m.buffers.to_device_act(cfg, w_gate_host) if gate else None

    w_exp = y_exp = None
    if experts:
        if w.dtype != workloads.BF16:
            print("bench.py: --experts needs a bf16 workload", file=sys.stderr)
            sys.exit(2)
        gen = torch.Generator(device="cuda").manual_seed(20_000 + w.seed)
        w_exp = torch.empty((w.experts, w.hidden, w.hidden), dtype=torch.bfloat16, device="cuda")
        for e in range(w.experts):          # expert by expert: the fp32 draws of all experts at once would not fit for every workload
            w_exp[e] = (torch.randn((w.hidden, w.hidden), generator=gen, device="cuda") / w.hidden ** 0.5).to(torch.bfloat16)
        y_exp = torch.empty_like(b.final)

    def step():
        if gate:
            m.monta_gate(cfg, b.x, w_gate, b.logits, stream)
        if experts:
            m.monta_route_dispatch_expert(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, w_exp, w.hidden, y_exp,
                                          b.ws, args.expert_overlap, stream)
            m.monta_combine(cfg, y_exp, b.gates, b.out, b.ws, stream)
            return
        m.monta_route_dispatch_regather(cfg, b.logits, b.x, b.topk_idx, b.gates, b.stage, b.final, b.ws, stream)
        if mirror:
            m.monta_unregather_combine(cfg, b.final, y_stage, b.gates, b.out, b.ws, stream)
        else:
            m.monta_combine(cfg, b.final, b.gates, b.out, b.ws, stream)

    torch.cuda.synchronize()
    use_graph = full and bool(args.graph)
    with torch.cuda.stream(stream):
        step()                              # first touch, also creates the side stream before any capture
        stream.synchronize()
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                step()
            run = graph.replay
        else:
            run = step
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    def time_eager(n):
        with torch.cuda.stream(stream):
            for _ in range(3):
                step()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(n):
                step()
            torch.cuda.synchronize()
            return (time.perf_counter() - c0) * 1e3 / n

    tabs = m.read_tables(cfg, b.ws)
    ab = algorithmic_bytes(w, tabs)
    if w.padded:
        pad_bytes = (tabs["final_rows"] - ab["R"]) * ab["row"]      # zero-filled by the regather of slice 0
        ab["total"] += pad_bytes
        ab["regather_s"][0] += pad_bytes
        ab["regather"] += pad_bytes
    if mirror:
        ab["total"] += 2 * ab["R"] * ab["row"]
        ab["unregather_s"] = ab["regather_s"]
        ab["combine_s"] = [ab["regather_s"][j] // 2 + (w.tokens // w.slices) * ab["row"] for j in range(w.slices)]
    if gate:
        ab["gate"] = (w.tokens + w.experts) * ab["row"] + w.tokens * w.experts * 4
        ab["total"] += ab["gate"]
    if experts:
        ab["expert_flops"] = 2.0 * ab["R"] * w.hidden * w.hidden
        ab["expert"] = (2 * ab["R"] + w.experts * w.hidden) * ab["row"]       # rows read and written once, weights once
        ab["total"] += ab["expert"]
    res = {"ms_per_step": ms_per_step, "ab": ab, "mode": mode, "use_graph": use_graph, "roofline": None, "kernels": {},
           "inputs": (logits, x), "w_gate_host": w_gate_host}
    if not full:
        del b
        return res

    # ---- per-kernel durations: HIP events around every launch, on the launching stream, eager launches
    kernels = {}
    if not args.no_profile:
        prof_steps = min(steps, 100)
        eager_ms = ms_per_step if not use_graph else time_eager(prof_steps)
        m.monta_profile_reset()
        m.monta_profile_enable(True)
        prof_ms = time_eager(prof_steps)
        m.monta_profile_enable(False)
        raw = {}
        for kid, name in enumerate(m.KERNEL_NAMES):
            ms, n = m.monta_profile_read(kid)
            if n:
                raw[name] = (ms, n)
        # Every timed interval holds one event marker.  What a marker costs in stream time is taken from
        # what the markers add to the step: (step with markers - step without) / markers per step.
        markers_per_step = sum(n for _, n in raw.values()) / (prof_steps + 3)
        marker_us = max(0.0, (prof_ms - eager_ms) * 1e3 / markers_per_step)
        for name, (ms, n) in raw.items():
            avg = ms * 1e3 / n - marker_us
            kernels[name] = {"launches_per_step": n / (prof_steps + 3), "avg_us": avg,
                             "us_per_step": avg * n / (prof_steps + 3)}
        m.monta_profile_reset()
        S = w.slices
        # bytes per launch of every kernel class, from the launch sequence the library reports for this problem
        pmode, first, spg, fused = m.monta_pipeline_query(cfg)
        groups = [range(0, first)] + [range(lo, min(lo + spg, S)) for lo in range(first, S, spg)]
        pack_g = [sum(ab["pack_s"][j] for j in gr) for gr in groups]
        reg_g = [sum(ab["regather_s"][j] for j in gr) for gr in groups]
        G = len(groups)
        seq = [("plan_pack" if fused else "pack", pack_g[0] + (ab["plan"] if fused else 0))]
        if pmode == 1:
            seq += [("pack_regather", pack_g[gi] + reg_g[gi - 1]) for gi in range(1, G)] + [("regather", reg_g[G - 1])]
        else:
            seq += [("regather", reg_g[0])]
            for gi in range(1, G):
                seq += [("pack", pack_g[gi]), ("regather", reg_g[gi])]
        per_launch = {"combine": ab["combine"], "gate": ab.get("gate")}
        for kname in ("pack", "regather", "pack_regather", "plan_pack"):
            vals = [v for n_, v in seq if n_ == kname]
            per_launch[kname] = sum(vals) / len(vals) if vals else None
        if experts and args.expert_overlap:      # the overlapped expert form runs the co-scheduled pipeline slice by slice
            per_launch["pack"] = ab["pack_s"][0]
            per_launch["regather"] = ab["regather_s"][S - 1]
            if S > 1:
                per_launch["pack_regather"] = sum(ab["pack_s"][j] + ab["regather_s"][j - 1] for j in range(1, S)) / (S - 1)
        if mirror:
            # the return pipeline: fetch and combine per launch group, as two kernels or co-scheduled; the group
            # count follows from the launches seen (groups are even)
            n_uc = round(kernels["unregather_combine"]["launches_per_step"]) if "unregather_combine" in kernels else 0
            Gm = n_uc + 1 if n_uc else max(1, round(kernels["unregather"]["launches_per_step"]))
            spg_m = -(-S // Gm)
            mgroups = [range(lo, min(lo + spg_m, S)) for lo in range(0, S, spg_m)]
            un_g = [sum(ab["unregather_s"][j] for j in gr) for gr in mgroups]
            cb_g = [sum(ab["combine_s"][j] for j in gr) for gr in mgroups]
            if n_uc:
                per_launch["unregather"] = un_g[0]
                per_launch["combine"] = cb_g[-1]
                per_launch["unregather_combine"] = sum(un_g[i] + cb_g[i - 1] for i in range(1, len(mgroups))) / n_uc
            else:
                per_launch["unregather"] = sum(un_g) / len(un_g)
                per_launch["combine"] = sum(cb_g) / len(cb_g)
        movers = [kname for kname in ("pack", "regather", "pack_regather", "combine", "plan_pack", "unregather",
                                      "unregather_combine", "gate") if kname in kernels]
        dom = max(movers, key=lambda kname: kernels[kname]["us_per_step"])
        achieved = per_launch[dom] / (kernels[dom]["avg_us"] * 1e-6) / 1e9
        # HBM-side bytes per launch of that kernel from rocprofv3 counters (profiles/traffic.json, written by
        # `python -m paper_2411_00662_amd.profiling traffic` from two --pmc runs of this same command)
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(tpath):
            try:
                entry = json.load(open(tpath)).get(f"{w.name}/S{w.slices}/mode{mode_label(mode)}", {})
                for kname, v in entry.items():
                    if kname.startswith(dom + "_kernel") or kname.startswith(dom + "_pf_kernel"):
                        traffic = v["total_bytes"]
            except (OSError, ValueError, KeyError):
                traffic = None
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                    "bytes_per_launch": int(per_launch[dom]), "avg_launch_us": round(kernels[dom]["avg_us"], 2),
                    "event_marker_us": round(marker_us, 2), "traffic": traffic}
        if "expert" in kernels:
            # the expert layer is a dense contraction: it is held against the matrix cores' bf16 peak
            ek = kernels["expert"]
            flops_per_launch = ab["expert_flops"] / max(1.0, ek["launches_per_step"])
            tflops = flops_per_launch / (ek["avg_us"] * 1e-6) / 1e12
            ek["TFLOPs"] = round(tflops, 1)
            if ek["us_per_step"] > kernels[dom]["us_per_step"]:
                roofline = {"bound": "mfma", "kernel": "expert", "achieved": round(tflops, 1),
                            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "flops_per_launch": int(flops_per_launch),
                            "avg_launch_us": round(ek["avg_us"], 2), "event_marker_us": round(marker_us, 2),
                            "traffic": None}
        for kname in movers:
            kernels[kname]["GBps"] = round(per_launch[kname] / (kernels[kname]["avg_us"] * 1e-6) / 1e9, 1)
        for v in kernels.values():
            for kk in list(v):
                v[kk] = round(v[kk], 3)
        res["roofline"] = roofline
        res["kernels"] = kernels
        res["pipeline"] = {"realisation": pmode, "first_launch_slices": first, "slices_per_launch": spg, "plan_fused_with_first_pack": fused}

    if args.calib_copy_mib > 0:
        nbytes = args.calib_copy_mib << 20
        src = torch.full((nbytes,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            m.monta_copy(dst, src, nbytes, stream)
        torch.cuda.synchronize()
        del src, dst
    del b
    return res


def cpu_baseline(args, w, res):
    """The CPU oracle on this host, on the whole workload: once on all cores (the OpenMP build of the same
    source) and once on one thread (the build the parity tests use).  Output arrays are allocated and touched by
    an untimed first pass, so the timed passes measure the oracle and not the host's page faults."""
    import oracle
    import workloads
    logits, x = res["inputs"]
    ab = res["ab"]
    kw = dict(k=w.top_k, ep=w.ep, tp=w.tp, S=w.slices, cf=w.capacity_factor, renorm=w.renorm, padded=w.padded)

    def one_pass(reuse):
        lg = oracle.gate(x, res["w_gate_host"]) if args.gate else logits
        return oracle.forward(lg, x, reuse=reuse, **kw)

    expert_s, expert_note = 0.0, ""
    with oracle.all_cores():
        cores = oracle.threads()
        ref = one_pass(None)             # untimed: allocates and touches STAGE / FINAL / out
        reps, spent = 0, 0.0
        while reps < 50 and spent < 8.0:
            c0 = time.perf_counter()
            one_pass(ref)
            spent += time.perf_counter() - c0
            reps += 1
    if args.experts:
        # the expert layer on a sample of rows of one expert, scaled to all kept rows (the whole layer would take hours)
        lo, hi = oracle.expert_ranges(ref.plan, w.tp, w.slices)
        e0 = int(np.argmax(hi - lo))
        n_rows = int(min(8, hi[e0] - lo[e0]))
        w_one = workloads.make_expert_weights(w.with_(experts=1))
        c0 = time.perf_counter()
        oracle.expert(ref.final[lo[e0]:lo[e0] + n_rows], w_one, np.array([0], np.int32), np.array([n_rows], np.int32))
        expert_s = (time.perf_counter() - c0) * ab["R"] / n_rows
        expert_note = f"; expert layer timed on {n_rows} rows on one thread and scaled to {ab['R']} ({expert_s:.0f} s per pass)"
    reps1, spent1 = 0, 0.0
    while reps1 < 50 and spent1 < 8.0:
        c0 = time.perf_counter()
        one_pass(ref)
        spent1 += time.perf_counter() - c0
        reps1 += 1
    per_pass, per_pass1 = spent / reps + expert_s, spent1 / reps1 + expert_s
    return {"value": round(w.tokens / per_pass, 1), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"the whole {w.name} workload, {reps} passes of the C oracle on {cores} threads ({spent:.1f} s)" + expert_note,
            "effective_GBps": round(ab["total"] / per_pass / 1e9, 2),
            "single_thread": {"value": round(w.tokens / per_pass1, 1), "unit": "tokens/s", "cores": 1,
                              "sample": f"the whole {w.name} workload, {reps1} passes on one thread ({spent1:.1f} s)",
                              "effective_GBps": round(ab["total"] / per_pass1 / 1e9, 2)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="skewed", help="tiny | mixtral | 2x70b | longctx | skewed (default: the largest)")
    ap.add_argument("--slices", type=int, default=0, help="override the workload's slice count")
    ap.add_argument("--mode", type=int, default=-1, help="pipeline realisation 0/1/2 (default -1: the library chooses)")
    ap.add_argument("--plan-mode", type=int, default=-1, help="how the plan tables are built: -1 library default, 0 ticketed scan")
    ap.add_argument("--graph", type=int, default=0, help="replay the step from a captured HIP graph (1) or launch eagerly (0)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run the plain copy kernel on buffers of this size (profiler byte-counter calibration)")
    ap.add_argument("--return-path", default="direct", choices=["direct", "mirror"],
                    help="direct: combine reads the expert output in FINAL layout (the headline path); mirror: the "
                         "second AllToAll mirrored (unregather + staged combine pipeline), 2R more rows moved")
    ap.add_argument("--padded", type=int, default=0, help="1: capacity-padded [E][C][H] layout of FINAL (zero-filled padding)")
    ap.add_argument("--gate", type=int, default=0,
                    help="1: the step starts one stage earlier, at the gate projection (monta_gate: logits = x * w_gate^T "
                         "with random-init weights); 0: at the logits, as the headline metric is defined")
    ap.add_argument("--experts", type=int, default=0,
                    help="1: a real expert layer (monta_route_dispatch_expert: one H x H linear layer per expert, random-init "
                         "weights) sits between dispatch and combine instead of identity experts")
    ap.add_argument("--expert-overlap", type=int, default=0,
                    help="with --experts 1: 1 = each slice's expert launch overlaps the next slice's movers (second stream)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other named workloads")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build covers one GPU's share of the path; nothing crosses GPUs, so only --gpus 1 is "
              "supported (virtual EP/TP ranks are buffer partitions on one MI355X).", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    import paper_2411_00662_amd as m

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    m.binding.lib()     # no fallback: fails here if the HIP library is not built

    w = workloads.CONFIGS[args.config]
    if args.slices:
        w = w.with_(slices=args.slices)
    if args.padded:
        w = w.with_(padded=1)
    m.monta_set_pipeline_mode(args.mode)
    m.monta_set_plan_mode(args.plan_mode)

    res = measure(args, w, args.steps, args.warmup, full=True)
    ms_per_step, ab = res["ms_per_step"], res["ab"]
    tokens_per_s = w.tokens / (ms_per_step * 1e-3)
    eff_gbps = ab["total"] / (ms_per_step * 1e-3) / 1e9

    # ---- CPU oracle on this host (a baseline for context, never the target)
    cpu = None if args.no_cpu else cpu_baseline(args, w, res)
    res.pop("inputs")
    gc.collect()
    torch.cuda.empty_cache()

    # ---- the other named workloads, briefly: step time and fraction of the HBM peak (headline path only)
    others = None
    plain = not (args.gate or args.experts or args.padded or args.slices or args.return_path != "direct")
    if not args.no_others and plain:
        others = {}
        for name in workloads.CONFIG_ORDER:
            if name == w.name:
                continue
            ow = workloads.CONFIGS[name]
            osteps = 200 if ow.tokens * ow.hidden <= 8192 * 8192 else 30        # short steps: more of them, so clocks settle
            r = measure(args, ow, osteps, 30 if osteps > 30 else 10, full=False)
            gb = r["ab"]["total"] / (r["ms_per_step"] * 1e-3) / 1e9
            others[name] = {"ms_per_step": round(r["ms_per_step"], 5),
                            "tokens_per_s": round(ow.tokens / (r["ms_per_step"] * 1e-3), 1),
                            "effective_GBps": round(gb, 1), "pct_of_hbm_peak": round(100 * gb / HBM_PEAK_GBPS, 2),
                            "kept_rows": r["ab"]["R"], "steps": osteps}
            r.clear()
            gc.collect()
            torch.cuda.empty_cache()

    line = {
        "metric": "dispatch+combine tokens/s", "value": round(tokens_per_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == workloads.BF16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "tokens": w.tokens, "hidden": w.hidden, "experts": w.experts,
                   "top_k": w.top_k, "ep": w.ep, "tp": w.tp, "slices": w.slices,
                   "capacity_factor": w.capacity_factor, "kept_rows": ab["R"], "alive_tokens": ab["alive"],
                   "pipeline_mode": mode_label(res["mode"]), "pipeline": res.get("pipeline"), "hip_graph": res["use_graph"], "return_path": args.return_path,
                   "padded": w.padded, "gate": bool(args.gate), "expert_layer": bool(args.experts),
                   "expert_overlap": int(args.expert_overlap), "parallelism": "1 GPU, virtual ep/tp"},
        "effective_GBps": round(eff_gbps, 1), "pct_of_hbm_peak": round(100 * eff_gbps / HBM_PEAK_GBPS, 2),
        "algorithmic_bytes_per_step": int(ab["total"]),
        "roofline": res["roofline"], "cpu_baseline": cpu, "other_configs": others, "kernels": res["kernels"],
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
