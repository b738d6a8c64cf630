#!/usr/bin/env python3
"""Benchmark of the hot path: one LSTM gradient step under the DP checkpoint policy.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--only] [--sweep | --fig2b | --chen]

A "step" is one call of ``mebptt_run``: every forward operation, every recomputation and every
backward operation of the schedule for one batch of synthetic sequences.  Inputs are resident in
device memory before the timed region.  Prints ONE JSON line on stdout (everything else goes to
stderr): throughput in time-steps/s at the named budget, the measured and theoretical cost
ratio against store-everything BPTT, the roofline position of the dominant kernel measured
with HIP events on the run's stream, and the CPU oracle timed on this host as a baseline.  Unless
--only is given the same line carries `configs` (every named configuration, a few steps each,
config 5 at each budget of its sweep) and `fig2b` (the shape of the paper's timing experiment).
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


def backward_bytes(w):
    """Algorithmic bytes of one backward operation's sequential half: W_hh once in the GEMM operand
    type, dG of the step after, the ten fp32 planes the pointwise step reads (h, c, four gates,
    c_prev, h_prev, dy, dc) and what it writes (dG twice -- row- and column-major -- h_prev
    transposed, dc)."""
    op = 2 if w.gemm_dtype else 4
    return (gate_blocks(w) * w.H * w.H * op + 4 * w.B * w.H * op + 40 * w.B * w.H
            + 2 * 4 * w.B * w.H * op + w.B * w.H * op + 4 * w.B * w.H)


def gate_blocks(w):
    """Gate blocks of the core's weight matrices: 4 (LSTM) or 3 (GRU)."""
    return 3 if w.cell else 4


def forward_flops(w):
    return 2 * gate_blocks(w) * w.B * w.H * (w.I + w.H)


def pmc_traffic(name="cfg2", kernel="forward_kernel"):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{name}_hbm_traffic.txt")
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


def memory_report(w, sess):
    """Bytes this run keeps against what store-everything BPTT would keep: the slot pool (the
    budget), the workspace outside it (working core, operand copies of the weights, dW accumulator,
    staging of two chunks), and t stored hidden or internal states in fp32."""
    plane = 4 * w.B * w.H
    return {"slot_pool_bytes": sess.slot_bytes, "workspace_bytes": sess.ws_bytes,
            "store_all_hidden_bytes": 2 * plane * w.t, "store_all_internal_bytes": 6 * plane * w.t,
            "pool_plus_workspace_over_store_all_internal": (sess.slot_bytes + sess.ws_bytes) / (6 * plane * w.t)}


def measure(w, inp, *, kind=None, m=None, steps=3, warmup=1, graph=True, profile=True, store_all=True,
            launch_floor_us=None, bracket_us=None, bracket_curve=None):
    """Times one configuration: ms per gradient step (stream launches and HIP-graph replay, the
    faster is reported), per kernel class the event-sampled time per launch and its MFMA fraction,
    the forward kernel's roofline position, the store-everything run for the cost ratio."""
    import torch
    from paper_1606_03401_amd import binding as mb
    from paper_1606_03401_amd import workloads as wl
    from paper_1606_03401_amd.session import Session
    sess = Session(w, inp, kind=kind, m=m, want_dx=True, want_y=False)
    ms = time_runs(sess, steps, warmup) * 1e3
    enqueue_ms = time_runs.last_enqueue_ms
    C = sess.plan.forward_ops
    eager_ms = ms
    graph_ms = time_graph(sess, steps, warmup) if graph else None
    launch_mode = "stream launches"
    if graph_ms is not None and graph_ms < ms:
        ms, launch_mode = graph_ms, "HIP graph replay"
    log(f"[bench] {w.name} {KIND_NAMES[sess.kind]} m={sess.m}: {ms:.3f} ms/step ({launch_mode}; host enqueue "
        f"{enqueue_ms:.3f} ms), forward ops {C}, peak {sess.plan.peak}")
    out = {"workload": f"{w.name}: single-layer {'GRU' if w.cell else 'LSTM'} I={w.I} H={w.H} B={w.B} t={w.t}, "
                       f"BPTT-{KIND_NAMES[sess.kind]} budget m={sess.m}, seed {w.seed}",
           "name": w.name, "kind": KIND_NAMES[sess.kind], "budget_m": sess.m, "forward_ops": C,
           "peak_slots": sess.plan.peak, "ms_per_step": ms, "ms_per_step_stream_launches": eager_ms,
           "ms_per_step_graph_replay": graph_ms, "launch": launch_mode, "host_enqueue_ms": enqueue_ms,
           "time_steps_per_s": w.t / (ms * 1e-3), "dtype": "bf16" if w.gemm_dtype else "f32",
           "memory": memory_report(w, sess)}
    flops_exec = (C + 2 * w.t) * forward_flops(w)
    peak_tf = MFMA_PEAK_TFLOPS[w.gemm_dtype]
    out["gflops"] = {"executed": flops_exec / (ms * 1e-3) / 1e9, "useful": 3 * w.t * forward_flops(w) / (ms * 1e-3) / 1e9,
                     "executed_frac_of_mfma_peak": flops_exec / (ms * 1e-3) / 1e12 / peak_tf}
    if profile:
        mb.mebptt_profile_enable(8)
        prof_steps = max(1, min(steps, 2))
        for _ in range(prof_steps):
            sess.run()
        torch.cuda.synchronize()
        prof = mb.mebptt_profile_collect()
        mb.mebptt_profile_enable(0)
        overhead_us = max(0.0, (bracket_us or 0.0) - (launch_floor_us or 0.0))

        def net_of(avg):
            """Event-bracketed time of a single launch -> that launch's own time, through the
            calibration curve (idle kernels of known length, bracketed and back to back)."""
            if not bracket_curve:
                return max(avg - overhead_us, 1e-3)
            pts = sorted(bracket_curve, key=lambda pb: pb[1])
            if avg <= pts[0][1]:
                return max(pts[0][0] - (pts[0][1] - avg), 1e-3)
            for (p0, b0), (p1, b1) in zip(pts, pts[1:]):
                if avg <= b1:
                    return p0 + (p1 - p0) * (avg - b0) / max(b1 - b0, 1e-9)
            return avg - (pts[-1][1] - pts[-1][0])
        # flops of one launch of each class: forward op 8BH(I+H); backward step (dh GEMM) 8BH^2; the
        # time-batched GEMMs carry t steps over their launches: dW 8BH(I+H), dx 8BHI per step.
        # The sequential GEMMs stream their weights once per launch: B flop per weight byte (bf16
        # operands: 2*B*K*N flop over 2*K*N bytes), so min(MFMA peak, B x HBM peak) is the most
        # such a launch can reach; the time-batched ones are bounded by the MFMA peak alone.
        F_fwd, F_dh = forward_flops(w), 2.0 * gate_blocks(w) * w.B * w.H * w.H
        F_dx = 2.0 * gate_blocks(w) * w.B * w.H * w.I
        opb = 2 if w.gemm_dtype else 4
        seq_cap_tf = min(peak_tf, 2.0 * w.B / opb * HBM_PEAK_GBS / 1e3)
        classes = {}
        for k, name in enumerate(mb.K_NAMES):
            n_s, n_g = prof.sampled[k], prof.sampled_groups[k]
            lps = prof.launches[k] / prof_steps
            avg_us = prof.sampled_ms[k] / n_s * 1e3 if n_s else None
            classes[name] = {"launches_per_step": lps, "avg_us": avg_us}
            if avg_us is not None and lps > 0:
                # a bracket holds n_s / n_g launches on average: its own time through the calibration
                # curve, then per launch (for the sequential classes this includes the gap between
                # dependent launches, as the chain pays it)
                per_group = n_s / max(n_g, 1)
                net_us = net_of(avg_us * per_group) / per_group
                flops = {"forward": F_fwd, "backward": F_dh, "backward+forward": F_dh + F_fwd,
                         "wgrad": w.t * F_fwd / lps, "dgrad": w.t * F_dx / lps,
                         "forward chain": F_fwd * prof.chain_steps / max(prof.launches[k], 1)}.get(name)
                classes[name]["net_us"] = net_us
                if flops:
                    tf = flops / (net_us * 1e-6) / 1e12
                    cap = peak_tf if name in ("wgrad", "dgrad") else seq_cap_tf
                    classes[name].update({"gflop_per_launch": flops / 1e9, "tflops": tf, "frac_mfma_peak": tf / peak_tf,
                                          "attainable_tflops": cap, "frac_of_attainable": tf / cap})
            log(f"[bench]   {name}: {lps:.0f} launches/step, avg {avg_us if avg_us is None else round(avg_us, 2)} us ({n_s} launches in {n_g} brackets)"
                + (f", net {classes[name]['net_us']:.2f} us, {classes[name]['tflops']:.0f} TFLOP/s = "
                   f"{100 * classes[name]['frac_mfma_peak']:.1f}% of MFMA peak, {100 * classes[name]['frac_of_attainable']:.0f}% of attainable"
                   if "tflops" in classes[name] else ""))
        out["kernel_classes"] = classes
        # Per-launch time of the sequential classes.  Forward launches: whole runs bracketed by one
        # event pair on the run's stream where there are any (single-launch brackets carry the cost
        # of the events themselves); forward chains: every launch bracketed, per carried step.
        if prof.forward_run_launches:
            classes["forward"]["net_us"] = prof.forward_run_ms / prof.forward_run_launches * 1e3
        if prof.chain_steps:
            ch = classes["forward chain"]
            ch["steps_per_step"] = prof.chain_steps / prof_steps
            ch["us_per_forward_op"] = prof.chain_ms / prof.chain_steps * 1e3
            log(f"[bench]   forward chain: {ch['steps_per_step']:.0f} forward ops/step in {ch['launches_per_step']:.0f} launches, "
                f"{ch['us_per_forward_op']:.2f} us per forward op")
        if prof.sweep_steps:
            sw = classes["sweep"]
            sw["steps_per_step"] = prof.sweep_steps / prof_steps
            sw["us_per_step"] = prof.sweep_ms / prof.sweep_steps * 1e3
            log(f"[bench]   sweep: {sw['steps_per_step']:.0f} backward steps/step in {sw['launches_per_step']:.0f} launches, "
                f"{sw['us_per_step']:.2f} us per step")
        if prof.batch_steps:
            fb = classes["forward batch"]
            fb["steps_per_step"] = prof.batch_steps / prof_steps
            fb["us_per_forward_op"] = prof.batch_ms / prof.batch_steps * 1e3
            log(f"[bench]   forward batch: {fb['steps_per_step']:.0f} independent forward ops/step in {fb['launches_per_step']:.0f} launches, "
                f"{fb['us_per_forward_op']:.2f} us per forward op")
        # The dominant kernel = the class with the largest share of the step; its roofline block.
        share = {}
        for name in ("forward", "backward", "backward+forward"):
            c = classes[name]
            if c.get("net_us") and c["launches_per_step"]:
                share[name] = c["net_us"] * c["launches_per_step"]
        if prof.chain_steps:
            share["forward chain"] = prof.chain_ms / prof_steps * 1e3
        if prof.sweep_steps:
            share["sweep"] = prof.sweep_ms / prof_steps * 1e3
        if prof.batch_steps:
            share["forward batch"] = prof.batch_ms / prof_steps * 1e3
        out["time_share_us"] = share
        if share:
            dom = max(share, key=share.get)
            kernel = {"forward": "forward_kernel", "backward": "backward_kernel", "backward+forward": "pair_kernel",
                      "forward chain": "forward_chain_kernel", "sweep": "sweep_kernel",
                      "forward batch": "forward_batch_kernel"}[dom]
            if dom == "sweep":
                # the weight operands stay on the chip; a step carries the dh GEMM and, in the launches
                # that recompute the internal state themselves, the forward GEMM as well
                us = classes[dom]["us_per_step"]
                fl = F_dh + F_fwd * prof.sweep_forward_steps / prof.sweep_steps
                tf = fl / (us * 1e-6) / 1e12
                out["roofline"] = {"bound": "mfma", "kernel": kernel, "achieved": tf, "peak": peak_tf, "unit": "TFLOP/s",
                                   "frac": tf / peak_tf, "traffic": None, "avg_launch_us": us,
                                   "flops_per_launch": fl, "note": "per backward step inside a sweep launch"}
            elif dom == "forward chain":
                # weights stay on the chip: what bounds a step is the matrix pipe and the exchange of h,
                # so the launch is placed on the MFMA roof
                us = classes[dom]["us_per_forward_op"]
                tf = forward_flops(w) / (us * 1e-6) / 1e12
                per_launch = pmc_traffic(w.name, kernel)   # HBM bytes of a whole chain launch (counter summary)
                ops_per_launch = prof.chain_steps / max(prof.launches[mb.K_CHAIN], 1)
                out["roofline"] = {"bound": "mfma", "kernel": kernel, "achieved": tf, "peak": peak_tf, "unit": "TFLOP/s",
                                   "frac": tf / peak_tf, "traffic": per_launch / ops_per_launch if per_launch else None,
                                   "traffic_per_chain_launch": per_launch, "avg_launch_us": us,
                                   "flops_per_launch": forward_flops(w), "note": "per forward operation inside a chain launch"}
            elif dom == "forward batch":
                # independent forward operations: a dense contraction over all their sequences at once
                us = classes[dom]["us_per_forward_op"]
                tf = forward_flops(w) / (us * 1e-6) / 1e12
                out["roofline"] = {"bound": "mfma", "kernel": kernel, "achieved": tf, "peak": peak_tf, "unit": "TFLOP/s",
                                   "frac": tf / peak_tf, "traffic": None, "avg_launch_us": us,
                                   "flops_per_launch": forward_flops(w), "note": "per forward operation inside a batch launch"}
            else:
                us = classes[dom]["net_us"]
                nbytes = {"forward": forward_bytes(w), "backward": backward_bytes(w),
                          "backward+forward": forward_bytes(w) + backward_bytes(w)}[dom]
                flops = {"forward": F_fwd, "backward": F_dh, "backward+forward": F_fwd + F_dh}[dom]
                achieved = nbytes / (us * 1e-6) / 1e9
                out["roofline"] = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
                                   "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": pmc_traffic(w.name, kernel),
                                   "avg_launch_us": us, "bytes_per_launch": nbytes,
                                   "mfma_tflops": flops / (us * 1e-6) / 1e12,
                                   "mfma_frac": flops / (us * 1e-6) / 1e12 / peak_tf}
    del sess
    store_all_ms = None
    if store_all:
        try:   # store-everything BPTT through the same path: an internal-state slot for every step
            sa = Session(w, inp, kind=wl.KIND_ISM, m=w.t, want_dx=True, want_y=False)
            store_all_ms = time_runs(sa, max(2, steps // 2), 1) * 1e3
            if graph and launch_mode == "HIP graph replay":
                g = time_graph(sa, max(2, steps // 2), 1)
                store_all_ms = min(store_all_ms, g) if g is not None else store_all_ms
            log(f"[bench]   store-all (ISM m=t): {store_all_ms:.3f} ms/step")
            del sa
        except Exception as e:   # e.g. the store-all pool does not fit
            log(f"[bench]   store-all run skipped: {e}")
    out["cost_ratio_vs_store_all"] = {"measured": (ms / store_all_ms) if store_all_ms else None,
                                      "theoretical": (C + 2 * w.t) / (3 * w.t), "store_all_ms": store_all_ms}
    return out


def fig2b_rows(steps, warmup, lengths=(100, 400, 1000)):
    """Section 4 / Fig. 2b as numbers: LSTM 256 -> 256, batch 64; microseconds per time step and
    forward operations per time step for budgets of 10/50/100/500/1000 hidden states and for
    store-everything BPTT, at several sequence lengths."""
    from paper_1606_03401_amd import workloads as wl
    from paper_1606_03401_amd.session import Session
    rows = []
    for t in lengths:
        base = wl.Workload("fig2b", B=64, I=256, H=256, t=t, kind=wl.KIND_HSM, m=t, gemm_dtype=wl.GEMM_BF16,
                           loss=wl.LOSS_EXTERNAL_DY, seed=t)
        inp = wl.make_inputs(base)
        row = {"t": t, "us_per_time_step": {}, "forward_ops_per_time_step": {}}
        for m in (10, 50, 100, 500, 1000):
            s = Session(base, inp, kind=wl.KIND_HSM, m=min(m, t), want_dx=True, want_y=False)
            row["us_per_time_step"][str(m)] = time_runs(s, steps, warmup) * 1e6 / t
            row["forward_ops_per_time_step"][str(m)] = s.plan.forward_ops / t
            del s
        sa = Session(base, inp, kind=wl.KIND_ISM, m=t, want_dx=True, want_y=False)
        row["us_per_time_step"]["store_all"] = time_runs(sa, steps, warmup) * 1e6 / t
        row["forward_ops_per_time_step"]["store_all"] = 1.0
        del sa
        rows.append(row)
        log(f"[fig2b] t={t}: " + "  ".join(f"m={k}: {v:.1f} us ({row['forward_ops_per_time_step'][k]:.2f} fwd)"
                                           for k, v in row["us_per_time_step"].items()))
    return rows


def floors(args) -> int:
    """The fixed costs the per-step times sit on, each measured alone on an otherwise idle device:
    a dependent empty launch, one synchronisation of a resident launch's workgroups (device-wide,
    per XCD, per XCD with the operand exchange), and the two time-batched GEMMs of one chunk for
    every named configuration."""
    import torch
    from paper_1606_03401_amd import binding as mb
    from paper_1606_03401_amd import workloads as wl
    out = {"experiment": "floors", "null_launch_us": mb.mebptt_null_launch_us(4000), "sync": [], "gemms_alone": []}
    log(f"[floors] dependent empty launch: {out['null_launch_us']:.2f} us")
    names = ("all 256 workgroups, one device-wide counter", "32 workgroups per XCD, per-XCD counter",
             "per-XCD counter + 16 KiB exchange through the L2")
    for v, name in enumerate(names):
        mb.mebptt_measure_sync(v, 200)   # warm-up
        us, status = mb.mebptt_measure_sync(v, 3000)
        out["sync"].append({"variant": v, "what": name, "us_per_sync": us, "status": status})
        log(f"[floors] sync variant {v} ({name}): {us:.2f} us, status {status}")
    for name in ("cfg2", "cfg3", "cfg4", "cfg5"):
        w = wl.CONFIGS[name]
        desc = mb.make_desc(w.B, w.I, w.H, w.t, w.gemm_dtype, w.loss, w.dy_first_step)
        ws = torch.zeros(mb.mebptt_workspace_bytes(desc), dtype=torch.uint8, device="cuda:0")
        su, sb = mb.mebptt_measure_forward_stream(desc, ws, 50)
        log(f"[floors] {name}: a kernel that only reads what a forward launch reads: {su:.2f} us per launch for {sb / 1e6:.0f} MB "
            f"through the L2s = {sb / su / 1e6:.1f} TB/s to the compute units (weights {forward_bytes(w) / 1e6:.1f} MB algorithmic)")
        wu, du = mb.mebptt_measure_gemms(desc, ws, 30)
        ch = mb.mebptt_chunk_steps(desc)
        fw, fd = ch * forward_flops(w), ch * 2.0 * gate_blocks(w) * w.B * w.H * w.I
        peak = MFMA_PEAK_TFLOPS[w.gemm_dtype]
        row = {"name": name, "forward_stream_us": su, "forward_stream_bytes": sb, "chunk_steps": ch, "wgrad_us": wu, "wgrad_tflops": fw / wu / 1e6, "wgrad_frac_mfma_peak": fw / wu / 1e6 / peak,
               "dgrad_us": du, "dgrad_tflops": fd / du / 1e6, "dgrad_frac_mfma_peak": fd / du / 1e6 / peak}
        out["gemms_alone"].append(row)
        log(f"[floors] {name}: chunk of {ch} steps: dW GEMM {wu:.1f} us = {row['wgrad_tflops']:.0f} TFLOP/s "
            f"({100 * row['wgrad_frac_mfma_peak']:.1f}% of MFMA peak); dx GEMM {du:.1f} us = {row['dgrad_tflops']:.0f} TFLOP/s "
            f"({100 * row['dgrad_frac_mfma_peak']:.1f}%)")
        del ws
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2", help="the configuration the headline value is measured on")
    ap.add_argument("--only", action="store_true", help="time the headline workload only (no `configs`, no `fig2b`)")
    ap.add_argument("--sweep", action="store_true", help="also time the budget sweep m = t .. 5%% of t on the headline shape")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time stream launches only")
    ap.add_argument("--fig2b", action="store_true",
                    help="only the shape of the paper's timing experiment: LSTM 256->256, batch 64, us per time step "
                         "vs sequence length at budgets of 10/50/100/500/1000 hidden states")
    ap.add_argument("--cell", choices=("lstm", "gru"), default="lstm", help="RNN core run on the workload's shape")
    ap.add_argument("--floors", action="store_true",
                    help="only the fixed costs: empty launch, workgroup synchronisation variants, the chunk GEMMs alone")
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

    if not torch.cuda.is_available():
        log("no GPU visible: the HIP path cannot run")
        return 1
    if args.fig2b:
        print(json.dumps({"experiment": "fig2b", "rows": fig2b_rows(args.steps, args.warmup, (100, 200, 400, 600, 800, 1000))}),
              flush=True)
        return 0
    if args.floors:
        return floors(args)
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
    # The floor of a dependent launch on this machine, and what an event pair around a single launch
    # adds to it (the low decile of brackets around a 4-byte fill): single-launch samples are
    # reported net of the difference.
    launch_floor_us = mb.mebptt_null_launch_us(4000)
    cal = torch.zeros(1, device="cuda:0")
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    for a, b in pairs:
        a.record()
        cal.zero_()
        b.record()
    torch.cuda.synchronize()
    bracket_us = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)[len(pairs) // 10]
    # What a bracket adds depends on how long the kernel inside it runs: idle kernels of known
    # length, timed back to back and each inside its own bracket, give the curve that turns an
    # event-sampled single-launch time into the launch's own time.
    bracket_curve = [mb.mebptt_bracket_overhead_us(L, 100) for L in (0, 2, 4, 8, 16, 32, 64)]
    log(f"[bench] back-to-back empty launches: {launch_floor_us:.2f} us each; event bracket around a minimal launch: "
        f"{bracket_us:.2f} us; bracket curve (own time -> bracketed): "
        + ", ".join(f"{a:.1f}->{b:.1f}" for a, b in bracket_curve))

    inp = wl.make_inputs(w)
    head = measure(w, inp, steps=args.steps, warmup=args.warmup, graph=not args.no_graph,
                   launch_floor_us=launch_floor_us, bracket_us=bracket_us, bracket_curve=bracket_curve)
    if args.sweep:
        from paper_1606_03401_amd.session import Session
        sa_ms = head["cost_ratio_vs_store_all"]["store_all_ms"]
        head["budget_sweep"] = []
        for kind in (wl.KIND_HSM, wl.KIND_ISM):
            for m in (w.t, w.t // 2, w.t // 4, w.t // 10, w.t // 20):
                s2 = Session(w, inp, kind=kind, m=m, want_dx=True, want_y=False)
                ms2 = time_runs(s2, max(2, args.steps // 2), 1) * 1e3
                Cm = s2.plan.forward_ops
                head["budget_sweep"].append({"kind": KIND_NAMES[kind], "m": m, "ms_per_step": ms2, "forward_ops": Cm,
                                             "theoretical_ratio": (Cm + 2 * w.t) / (3 * w.t),
                                             "measured_ratio": ms2 / sa_ms if sa_ms else None})
                log(f"[sweep] {KIND_NAMES[kind]} m={m}: {ms2:.3f} ms, {w.t / ms2 * 1e3:.0f} steps/s, C={Cm}, "
                    f"theoretical ratio {(Cm + 2 * w.t) / (3 * w.t):.3f}, measured {ms2 / sa_ms if sa_ms else float('nan'):.3f}")
                del s2
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, inp, 12.0 if not args.only else 20.0)
        log(f"[bench] cpu baseline {cpu}")
    del inp

    ms = head["ms_per_step"]
    result = {
        "metric": METRIC, "value": w.t / (ms * 1e-3), "unit": "time-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "ms_per_step_stream_launches": head["ms_per_step_stream_launches"], "ms_per_step_graph_replay": head["ms_per_step_graph_replay"],
        "host_enqueue_ms": head["host_enqueue_ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "launch": head["launch"], "budget_m": head["budget_m"],
                   "forward_ops": head["forward_ops"], "peak_slots": head["peak_slots"],
                   "slot_pool_bytes": head["memory"]["slot_pool_bytes"], "workspace_bytes": head["memory"]["workspace_bytes"]},
        "cost_ratio_vs_store_all": head["cost_ratio_vs_store_all"],
        "gflops": head["gflops"],
        "launch_floor_us": launch_floor_us, "event_bracket_us": bracket_us,
        "kernel_classes": head.get("kernel_classes"),
        "roofline": head.get("roofline"),
        "memory": head["memory"],
    }
    if "budget_sweep" in head:
        result["budget_sweep"] = head["budget_sweep"]
    if cpu is not None:
        result["cpu_baseline"] = cpu

    if not args.only:
        # Every other configuration, a few steps each (cfg5 at each budget of its sweep), with the
        # same per-class and roofline figures and a short CPU-oracle sample of its own.
        configs = [dict(head, cpu_baseline=cpu)]
        for name in ("cfg1", "cfg3", "cfg4", "cfg5"):
            if name == args.workload:
                continue
            wc = wl.CONFIGS[name]
            inp_c = wl.make_inputs(wc)
            budgets = wl.CFG5_BUDGET_SWEEP if name == "cfg5" else (wc.m,)
            for i, m in enumerate(budgets):
                few = 2 if (name == "cfg5" and m < 31) else 3
                row = measure(wc, inp_c, m=m, steps=few, warmup=1, graph=not args.no_graph,
                              profile=(m == wc.m), store_all=(i == 0),
                              launch_floor_us=launch_floor_us, bracket_us=bracket_us, bracket_curve=bracket_curve)
                if i > 0:   # one store-everything run serves the whole sweep
                    sa_ms = configs[-i]["cost_ratio_vs_store_all"]["store_all_ms"]
                    row["cost_ratio_vs_store_all"].update({"store_all_ms": sa_ms,
                                                           "measured": row["ms_per_step"] / sa_ms if sa_ms else None})
                if m == wc.m and not args.no_cpu_baseline:
                    row["cpu_baseline"] = cpu_baseline(wc, inp_c, 4.0)
                    log(f"[bench]   cpu baseline {row['cpu_baseline']}")
                configs.append(row)
            del inp_c
        result["configs"] = configs
        result["fig2b"] = {"shape": "LSTM I=256 H=256 B=64, bf16 GEMM operands, HSM budgets and store-all",
                           "rows": fig2b_rows(3, 1)}
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
