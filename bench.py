#!/usr/bin/env python3
"""Benchmark of the hot path: one LSTM gradient step under the DP checkpoint policy.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--sweep | --fig2b | --chen]

A "step" is one call of ``mebptt_run``: every forward operation, every recomputation and every
backward operation of the schedule for one batch of synthetic sequences.  Inputs are resident in
device memory before the timed region.  Prints ONE JSON line on stdout (everything else goes to
stderr): throughput in time-steps/s at the named budget, the measured and theoretical cost
ratio against store-everything BPTT, the roofline position of the dominant kernel measured
with HIP events on the run's stream, and the CPU oracle timed on this host as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "LSTM BPTT time-steps/s at budget m; cost ratio vs store-all BPTT"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
MFMA_PEAK_TFLOPS = {0: 157.3, 1: 2500.0}   # by gemm_dtype: fp32 operands, bf16 operands
KIND_NAMES = {0: "HSM", 1: "ISM", 2: "MSM"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_runs(sess, steps, warmup):
    import torch
    for _ in range(warmup):
        sess.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    enq = 0.0
    for _ in range(steps):
        e0 = time.perf_counter()
        sess.run()
        enq += time.perf_counter() - e0
    torch.cuda.synchronize()
    time_runs.last_enqueue_ms = enq / steps * 1e3      # host time spent inside mebptt_run (enqueue only)
    return (time.perf_counter() - t0) / steps


def time_graph(sess, steps, warmup):
    """The schedule is static, so the same launches can be replayed from a HIP graph; this removes
    the per-launch host cost (it matters when the host, not the GPU, is the limit)."""
    import torch
    try:
        sess.capture()
        for _ in range(warmup):
            sess.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            sess.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        log(f"[bench] HIP graph replay: {ms:.3f} ms/step")
        return ms
    except Exception as e:
        log(f"[bench] graph capture skipped: {e}")
        return None


def forward_bytes(w):
    """Algorithmic bytes of one forward operation: the gate weights once in the GEMM operand
    type, x_t once, and the hidden state (h, c) read and written once in fp32."""
    op = 2 if w.gemm_dtype else 4
    return gate_blocks(w) * w.H * (w.I + w.H) * op + 4 * w.B * w.I + 16 * w.B * w.H


def gate_blocks(w):
    """Gate blocks of the core's weight matrices: 4 (LSTM) or 3 (GRU)."""
    return 3 if w.cell else 4


def forward_flops(w):
    return 2 * gate_blocks(w) * w.B * w.H * (w.I + w.H)


def pmc_traffic():
    """HBM bytes per forward launch from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "forward_kernel_cfg2_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(w, inp, budget_s=20.0):
    """The oracle (float64 store-everything BPTT) on this host, on a prefix of the workload's
    sequence sized to take roughly `budget_s` seconds."""
    import numpy as np
    from oracle import gru_bptt as og
    from oracle import lstm_bptt as ob
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    probe = min(8, w.t)

    def run(n):
        dy = None if inp.dy is None else inp.dy[:max(0, n - w.dy_first_step + 1)]
        first = min(w.dy_first_step, n)
        if inp.dy is not None and dy.shape[0] == 0:
            dy, first = np.zeros((1,) + inp.dy.shape[1:], np.float32), n
        t0 = time.perf_counter()
        if w.cell:
            og.gru_bptt(inp.W_ih, inp.W_hh, inp.b, inp.x[:n], inp.h0, dy, first)
        else:
            ob.lstm_bptt(inp.W_ih, inp.W_hh, inp.b, inp.x[:n], inp.h0, inp.c0, dy, first)
        return time.perf_counter() - t0

    per_step = run(probe) / probe
    n = int(max(probe, min(w.t, budget_s / max(per_step, 1e-9))))
    dt = run(n)
    return {"value": n / dt, "unit": "time-steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n} of {w.t} steps of {w.name} (float64 store-everything BPTT, numpy), {dt:.1f} s"}


def fig2b(args) -> int:
    """Section 4 / Fig. 2b: time per time step of one gradient step as a function of the sequence
    length, for budgets of 10, 50, 100, 500, 1000 hidden states, beside the cost model's forward
    operations per step (Fig. 2a).  Synthetic inputs; the paper states no hardware or precision."""
    import torch
    from paper_1606_03401_amd import workloads as wl
    from paper_1606_03401_amd.session import Session
    rows = []
    for t in (100, 200, 400, 600, 800, 1000):
        base = wl.Workload("fig2b", B=64, I=256, H=256, t=t, kind=wl.KIND_HSM, m=t, gemm_dtype=wl.GEMM_BF16,
                           loss=wl.LOSS_EXTERNAL_DY, seed=t)
        inp = wl.make_inputs(base)
        line = {"t": t}
        for m in (10, 50, 100, 500, 1000):
            s = Session(base, inp, kind=wl.KIND_HSM, m=min(m, t), want_dx=True, want_y=False)
            ms = time_runs(s, args.steps, args.warmup) * 1e3
            line[m] = (ms / t * 1e3, s.plan.forward_ops / t)
            del s
        sa = Session(base, inp, kind=wl.KIND_ISM, m=t, want_dx=True, want_y=False)
        line["store_all"] = (time_runs(sa, args.steps, args.warmup) * 1e3 / t * 1e3, 1.0)
        del sa
        rows.append(line)
        log(f"[fig2b] t={t}: " + "  ".join(
            f"m={k}: {v[0]:.1f} us/step ({v[1]:.2f} fwd/step)" for k, v in line.items() if k != "t"))
    print(json.dumps({"experiment": "fig2b", "unit": "us per time step (forward ops per step)", "rows": rows}), flush=True)
    return 0


def chen_comparison(args) -> int:
    """Sections 4.2-4.3: Chen et al.'s sqrt(t) and recursive strategies run as policies through the
    same executor on the benchmark workload, beside the optimal BPTT-MSM policy at the same memory,
    and the two quantities of the paper's numerical comparison computed from the planner's tables
    (memory needed for a cost of 2 forward operations per step relative to sqrt(t)(1+beta), and
    cost per step at that memory; alpha = beta + 1)."""
    import math
    from paper_1606_03401_amd import binding as mb
    from paper_1606_03401_amd import workloads as wl
    from paper_1606_03401_amd.session import Session
    w = wl.CONFIGS[args.workload]
    inp = wl.make_inputs(w)
    rows = []
    cases = [("chen sqrt(t)", mb.mebptt_plan_chen_sqrt(w.t))]
    cases += [(f"chen recursive k={k}", mb.mebptt_plan_chen_recursive(w.t, k)) for k in (1, 2, 4, 9)]
    for name, plan in cases:
        for label, pl in ((name, plan), (f"  BPTT-MSM at the same {plan.m} units", mb.mebptt_plan(w.t, plan.m, mb.MSM))):
            sess = Session(w, inp, plan=pl, want_dx=True, want_y=False)
            ms = time_runs(sess, args.steps, args.warmup) * 1e3
            rows.append({"strategy": label.strip(), "units": pl.m, "slot_MiB": sess.slot_bytes / 2**20,
                         "forward_ops": pl.forward_ops, "ms_per_step": ms})
            log(f"[chen] {label:42s} {pl.m:5d} units ({sess.slot_bytes / 2**20:7.1f} MiB)  C = {pl.forward_ops:6d} "
                f"({pl.forward_ops / w.t:.3f}/step)  {ms:8.3f} ms")
            del sess
    fig = []
    for beta in (2, 5, 10):
        for t in (100, 400, 1000):
            ref = math.sqrt(t) * (1 + beta)
            m_ref = int(ref)
            tab = mb.mebptt_plan(t, m_ref, mb.MSM, beta + 1, beta)   # tables only (alpha may be below 4)
            C = tab.cost(0)[t]
            m_cost2 = next(m for m in range(1, m_ref + 1) if C[m] <= 2 * t)
            fig.append({"beta": beta, "t": t, "memory_ratio_at_cost_2": m_cost2 / ref, "cost_per_step_at_chen_memory": C[m_ref] / t})
            log(f"[chen] beta={beta:2d} t={t:4d}: memory at cost 2 = {m_cost2:4d} units = {m_cost2 / ref:.3f} x sqrt(t)(1+beta); "
                f"cost at sqrt(t)(1+beta) = {C[m_ref] / t:.3f} per step")
    print(json.dumps({"experiment": "chen", "workload": w.name, "rows": rows, "section_4_3": fig}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--sweep", action="store_true", help="also time the budget sweep m = t .. 5%% of t (stderr)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time stream launches only")
    ap.add_argument("--fig2b", action="store_true",
                    help="the shape of the paper's timing experiment: LSTM 256->256, batch 64, ms per time step "
                         "vs sequence length at budgets of 10/50/100/500/1000 hidden states (table on stderr)")
    ap.add_argument("--cell", choices=("lstm", "gru"), default="lstm", help="RNN core run on the workload's shape")
    ap.add_argument("--chen", action="store_true",
                    help="Chen et al.'s sqrt(t) / recursive strategies as policies through the same executor, beside "
                         "BPTT-MSM at the same memory, and the paper's numerical comparison (table on stderr)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: this build runs the path on a single device; --gpus must be 1")
        return 2

    import torch
    from paper_1606_03401_amd import binding as mb
    from paper_1606_03401_amd import workloads as wl
    from paper_1606_03401_amd.session import Session

    if not torch.cuda.is_available():
        log("no GPU visible: the HIP path cannot run")
        return 1
    if args.fig2b:
        return fig2b(args)
    if args.chen:
        return chen_comparison(args)
    w = wl.CONFIGS[args.workload]
    if args.cell == "gru":
        w = w.scaled(name=w.name + "-gru", cell=wl.CELL_GRU)
    log(f"[bench] {mb.mebptt_version()} workload {w}")
    # A plain device-to-device copy of known size (256 MiB read + 256 MiB written): the yardstick
    # that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters into bytes (see profiles/).
    cal_src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    inp = wl.make_inputs(w)
    sess = Session(w, inp, want_dx=True, want_y=False)
    ms = time_runs(sess, args.steps, args.warmup) * 1e3
    C = sess.plan.forward_ops
    enqueue_ms = time_runs.last_enqueue_ms
    log(f"[bench] {KIND_NAMES[sess.kind]} m={sess.m}: {ms:.3f} ms/step (host enqueue {enqueue_ms:.3f} ms), "
        f"forward ops {C}, peak {sess.plan.peak}")
    eager_ms = ms
    graph_ms = None if args.no_graph else time_graph(sess, args.steps, args.warmup)
    launch_mode = "stream launches"
    if graph_ms is not None and graph_ms < ms:
        ms, launch_mode = graph_ms, "HIP graph replay"

    # dominant kernel: event-bracketed samples on the run's stream, in extra profiled steps
    mb.mebptt_profile_enable(8)
    prof_steps = max(1, min(args.steps, 3))
    for _ in range(prof_steps):
        sess.run()
    torch.cuda.synchronize()
    prof = mb.mebptt_profile_collect()
    mb.mebptt_profile_enable(0)
    # What an event pair around a single launch adds: the same bracket around a launch that does
    # nothing measurable (a 4-byte fill), minus nothing -- an upper bound of the bracket's own cost.
    cal = torch.zeros(1, device=sess.dev)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    for a, b in pairs:
        a.record()
        cal.zero_()
        b.record()
    torch.cuda.synchronize()
    bracket_us = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)[len(pairs) // 10]   # low decile: the bracket's floor
    null_us = 2.4   # a back-to-back empty launch on this stack: part of every kernel's own time
    overhead_us = max(0.0, bracket_us - null_us)
    log(f"[bench] event bracket around a minimal launch: {bracket_us:.2f} us -> {overhead_us:.2f} us subtracted from single-launch samples")
    # flops of one launch of each class: forward op 8BH(I+H); backward step (dh GEMM) 8BH^2; the
    # time-batched GEMMs carry t steps over their launches: dW 8BH(I+H), dx 8BHI per step
    F_fwd, F_dh = forward_flops(w), 2.0 * gate_blocks(w) * w.B * w.H * w.H
    F_dx = 2.0 * gate_blocks(w) * w.B * w.H * w.I
    classes = {}
    for k, name in enumerate(mb.K_NAMES):
        n_s = prof.sampled[k]
        lps = prof.launches[k] / prof_steps
        avg_us = prof.sampled_ms[k] / n_s * 1e3 if n_s else None
        classes[name] = {"launches_per_step": lps, "avg_us": avg_us}
        if avg_us is not None and lps > 0:
            net_us = max(avg_us - overhead_us, 1e-3)
            flops = {"forward": F_fwd, "backward": F_dh, "backward+forward": F_dh + F_fwd,
                     "wgrad": w.t * F_fwd / lps, "dgrad": w.t * F_dx / lps}.get(name)
            classes[name]["net_us"] = net_us
            if flops:
                tf = flops / (net_us * 1e-6) / 1e12
                classes[name].update({"gflop_per_launch": flops / 1e9, "tflops": tf, "frac_mfma_peak": tf / MFMA_PEAK_TFLOPS[w.gemm_dtype]})
        log(f"[bench] kernel class {name}: {lps:.0f} launches/step, "
            f"avg {avg_us if avg_us is None else round(avg_us, 2)} us (event-bracketed, {n_s} samples)"
            + (f", net {classes[name]['net_us']:.2f} us, {classes[name]['tflops']:.0f} TFLOP/s = "
               f"{100 * classes[name]['frac_mfma_peak']:.1f}% of MFMA peak" if "tflops" in classes[name] else ""))
    # The dominant kernel's launch duration: whole forward runs bracketed by one event pair (the
    # figure rocprofv3's kernel trace reports); single-launch brackets carry ~4 us of event cost.
    if prof.forward_run_launches:
        fwd_us = prof.forward_run_ms / prof.forward_run_launches * 1e3
        log(f"[bench] forward kernel inside long runs: avg {fwd_us:.2f} us over {prof.forward_run_launches} launches")
    else:
        fwd_us = classes["forward"]["avg_us"]
    achieved = forward_bytes(w) / (fwd_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": "forward_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": pmc_traffic(),
                "avg_launch_us": fwd_us, "bytes_per_launch": forward_bytes(w),
                "mfma_tflops": forward_flops(w) / (fwd_us * 1e-6) / 1e12,
                "mfma_frac": forward_flops(w) / (fwd_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS}

    # store-everything BPTT through the same path: internal-state slots for every step
    store_all_ms = None
    try:
        sa = Session(w, inp, kind=wl.KIND_ISM, m=w.t, want_dx=True, want_y=False)
        store_all_ms = time_runs(sa, max(2, args.steps // 2), 1) * 1e3
        if launch_mode == "HIP graph replay":
            g = time_graph(sa, max(2, args.steps // 2), 1)
            store_all_ms = min(store_all_ms, g) if g is not None else store_all_ms
        log(f"[bench] store-all (ISM m=t): {store_all_ms:.3f} ms/step, forward ops {sa.plan.forward_ops}")
        del sa
    except Exception as e:   # e.g. the store-all pool does not fit
        log(f"[bench] store-all run skipped: {e}")

    if args.sweep:
        for kind in (wl.KIND_HSM, wl.KIND_ISM):
            for m in (w.t, w.t // 2, w.t // 4, w.t // 10, w.t // 20):
                s2 = Session(w, inp, kind=kind, m=m, want_dx=True, want_y=False)
                ms2 = time_runs(s2, max(2, args.steps // 2), 1) * 1e3
                Cm = s2.plan.forward_ops
                log(f"[sweep] {KIND_NAMES[kind]} m={m}: {ms2:.3f} ms, {w.t / ms2 * 1e3:.0f} steps/s, C={Cm}, "
                    f"theoretical ratio {(Cm + 2 * w.t) / (3 * w.t):.3f}, "
                    f"measured {ms2 / store_all_ms if store_all_ms else float('nan'):.3f}")
                del s2

    flops_exec = (C + 2 * w.t) * forward_flops(w)
    flops_useful = 3 * w.t * forward_flops(w)
    result = {
        "metric": METRIC, "value": w.t / (ms * 1e-3), "unit": "time-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "ms_per_step_stream_launches": eager_ms, "ms_per_step_graph_replay": graph_ms,
        "host_enqueue_ms": enqueue_ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.gemm_dtype else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: single-layer {'GRU' if w.cell else 'LSTM'} I={w.I} H={w.H} B={w.B} t={w.t}, "
                               f"BPTT-{KIND_NAMES[sess.kind]} budget m={sess.m}, seed {w.seed}",
                   "launch": launch_mode, "budget_m": sess.m, "forward_ops": C, "peak_slots": sess.plan.peak,
                   "slot_pool_bytes": sess.slot_bytes, "workspace_bytes": sess.ws_bytes},
        "cost_ratio_vs_store_all": {"measured": (ms / store_all_ms) if store_all_ms else None,
                                    "theoretical": (C + 2 * w.t) / (3 * w.t), "store_all_ms": store_all_ms},
        "gflops": {"executed": flops_exec / (ms * 1e-3) / 1e9, "useful": flops_useful / (ms * 1e-3) / 1e9,
                   "executed_frac_of_mfma_peak": flops_exec / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "kernel_classes": classes,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, inp)
        log(f"[bench] cpu baseline {result['cpu_baseline']}")
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
