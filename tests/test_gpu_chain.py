"""GPU tests of the forward-chain and sweep launches (a chain of forward operations, or a run of
forward+backward pairs, in one launch, weights resident on the chip, the batch split over the
XCDs): against the float64 oracle, bit for
bit against the launch-per-step path on the same inputs, for every strategy and many budgets, on
every shape class the kernel is instantiated for, with ragged batches, and from two host threads
at once."""
import threading

import numpy as np
import pytest

from oracle import lstm_bptt as ob
from paper_1606_03401_amd import binding as mb
from paper_1606_03401_amd import workloads as wl

pytestmark = pytest.mark.gpu

FIELDS = ("dW_ih", "dW_hh", "db", "dh0", "dc0", "dx", "y")


def _same(a, b, what=""):
    for f in FIELDS:
        assert np.array_equal(getattr(a, f), getattr(b, f)), (what, f)


def _run(w, inp, kind, m, chain):
    from paper_1606_03401_amd.session import Session
    mb.mebptt_forward_chain_enable(chain)
    try:
        s = Session(w, inp, kind=kind, m=m)
        out = s.run_and_fetch()          # raises if a chain launch gave up
    finally:
        mb.mebptt_forward_chain_enable(True)
    return out


SHAPES = [
    # B, I, H, t: (H/128, steps per wave, K split, batch tiles per XCD) in the comment
    (64, 128, 128, 40),     # (1, 2, 4, 1)
    (37, 100, 128, 33),     # (1, 2, 4, 2): ragged batch, groups straddle tiles, ragged I
    (5, 128, 128, 20),      # fewer sequences than XCDs
    (64, 256, 256, 60),     # (2, 4, 4, 1): the paper's experiment
    (150, 250, 256, 25),    # (2, 4, 4, 2)
    (256, 128, 512, 30),    # (4, 5, 4, 2): configuration 4's shape
    (100, 128, 512, 30),    # (4, 5, 4, 1)
    (64, 256, 1024, 60),    # (8, 5, 8, 1): configuration 2's shape
    (40, 250, 1024, 20),    # same class, ragged batch and input width
]


@pytest.mark.parametrize("B,I,H,t", SHAPES)
def test_chain_matches_per_step_path_and_oracle(B, I, H, t):
    from test_gpu_parity import TOL, check_against_oracle
    w = wl.Workload("chain", B=B, I=I, H=H, t=t, kind=wl.KIND_HSM, m=4, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, dy_first_step=2, seed=900 + B + H)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    ref = ob.lstm_bptt(inp.W_ih, inp.W_hh, inp.b, inp.x, inp.h0, inp.c0, inp.dy, w.dy_first_step)
    base = _run(w, inp, wl.KIND_HSM, 3, chain=False)
    check_against_oracle(w, inp, base, ref, TOL[w.gemm_dtype], label=f"chain {B}x{I}x{H} per-step: ")
    cases = [(wl.KIND_HSM, 1), (wl.KIND_HSM, 2), (wl.KIND_HSM, 3), (wl.KIND_HSM, 7), (wl.KIND_HSM, t),
             (wl.KIND_ISM, 1), (wl.KIND_ISM, 3), (wl.KIND_ISM, t), (wl.KIND_MSM, 2), (wl.KIND_MSM, 9), (wl.KIND_MSM, 4 * t)]
    for kind, m in cases:
        out = _run(w, inp, kind, m, chain=True)
        _same(out, base, (kind, m))
        assert out.stats.backward_ops == t


def test_chain_launch_count_and_status():
    """The launches really are chains: with the chain path on, a store-everything HSM plan of a
    long sequence needs far fewer forward launches than forward operations, and the status word
    stays clear."""
    from paper_1606_03401_amd.session import Session
    w = wl.Workload("chain-count", B=64, I=128, H=128, t=200, kind=wl.KIND_HSM, m=200, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, seed=31)
    inp = wl.make_inputs(w)
    s = Session(w, inp)
    mb.mebptt_profile_enable(1)
    out = s.run_and_fetch()
    prof = mb.mebptt_profile_collect()
    mb.mebptt_profile_enable(0)
    assert mb.mebptt_run_status(s.desc, s.workspace) == 0
    assert out.stats.forward_ops == 2 * w.t - 1
    assert prof.chain_steps >= w.t - 2                     # the initial forward pass went out as chains
    assert prof.launches[mb.K_CHAIN] <= (w.t + 47) // 48 + 1
    assert prof.sweep_steps >= w.t - 40                    # and the way back as sweep launches, one per chunk of steps
    assert prof.launches[mb.K_SWEEP] <= (w.t + 31) // 32 + 1
    assert prof.sweep_forward_steps == prof.sweep_steps    # these sweep launches recompute the internal states themselves
    assert (prof.launches[mb.K_FORWARD] + prof.launches[mb.K_PAIR] + prof.chain_steps + prof.sweep_forward_steps
            + prof.batch_steps == out.stats.forward_ops)
    assert prof.launches[mb.K_BACKWARD] + prof.launches[mb.K_PAIR] + prof.sweep_steps == w.t
    # store-everything BPTT (an internal-state slot per step): the forward pass as chains, the backward pass
    # through the stored states as backward-only sweep launches
    s2 = Session(w, inp, kind=wl.KIND_ISM, m=w.t)
    mb.mebptt_profile_enable(1)
    out2 = s2.run_and_fetch()
    prof2 = mb.mebptt_profile_collect()
    mb.mebptt_profile_enable(0)
    assert out2.stats.forward_ops == w.t and prof2.chain_steps >= w.t - 2 and prof2.sweep_forward_steps == 0
    assert prof2.sweep_steps >= w.t - 40 and prof2.launches[mb.K_BACKWARD] + prof2.sweep_steps == w.t
    for f in FIELDS:
        assert np.array_equal(getattr(out2, f), getattr(out, f)), f


@pytest.mark.parametrize("B,I,H,t", [(64, 256, 1024, 70), (64, 120, 1024, 45), (128, 64, 1024, 40), (16, 30, 1024, 37), (100, 120, 1024, 45)])
def test_batched_recomputation(B, I, H, t):
    """H = 1024: the weights of both directions do not fit on the chip together, so the way back
    through a stretch of stored hidden states is one launch of independent forward operations (the
    internal states of up to a chunk of steps, into the stage) followed by one backward-only sweep
    launch.  The launches really are those, every forward operation is accounted for, and the
    gradients are the per-step path's bit for bit and the oracle's within tolerance."""
    from paper_1606_03401_amd.session import Session
    from test_gpu_parity import TOL, check_against_oracle
    w = wl.Workload("batch", B=B, I=I, H=H, t=t, kind=wl.KIND_HSM, m=t, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, dy_first_step=3, seed=400 + B)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    ref = ob.lstm_bptt(inp.W_ih, inp.W_hh, inp.b, inp.x, inp.h0, inp.c0, inp.dy, w.dy_first_step)
    base = _run(w, inp, wl.KIND_HSM, t, chain=False)
    for kind, m in ((wl.KIND_HSM, t), (wl.KIND_HSM, 9), (wl.KIND_HSM, 4), (wl.KIND_MSM, 30), (wl.KIND_ISM, t)):
        s = Session(w, inp, kind=kind, m=m)
        mb.mebptt_profile_enable(1)
        out = s.run_and_fetch()
        prof = mb.mebptt_profile_collect()
        mb.mebptt_profile_enable(0)
        assert mb.mebptt_run_status(s.desc, s.workspace) == 0
        _same(out, base, ("batched recomputation", kind, m))
        assert prof.sweep_forward_steps == 0 and prof.sweep_steps > 0
        assert prof.launches[mb.K_FWD_BATCH] <= prof.launches[mb.K_SWEEP]
        assert (prof.launches[mb.K_FORWARD] + prof.launches[mb.K_PAIR] + prof.chain_steps + prof.batch_steps
                == out.stats.forward_ops)
        assert prof.launches[mb.K_BACKWARD] + prof.launches[mb.K_PAIR] + prof.sweep_steps == t
        if kind == wl.KIND_HSM:   # a sweep launch may start with a step whose state a forward run left in the core
            assert prof.batch_steps <= prof.sweep_steps <= prof.batch_steps + prof.launches[mb.K_SWEEP]
        if kind == wl.KIND_HSM and m == t:
            assert prof.batch_steps >= t - 8     # all but single steps left over at chunk boundaries
        if kind == wl.KIND_ISM:
            assert prof.batch_steps == 0         # the internal states were stored on the way forward
    check_against_oracle(w, inp, base, ref, TOL[w.gemm_dtype], label=f"batched recomputation {B}x{I}x{H}: ")


def test_chains_from_two_host_threads():
    """Two host threads with their own streams run chain-eligible workloads at the same time: the
    library orders the two runs on the device (each chain launch wants the whole chip) and both
    give the single-threaded result."""
    import torch
    from paper_1606_03401_amd.session import Session
    ws = [wl.Workload("cthr-a", B=64, I=128, H=128, t=90, kind=wl.KIND_HSM, m=6, gemm_dtype=wl.GEMM_BF16,
                      loss=wl.LOSS_EXTERNAL_DY, seed=81),
          wl.Workload("cthr-b", B=64, I=256, H=256, t=70, kind=wl.KIND_MSM, m=12, gemm_dtype=wl.GEMM_BF16,
                      loss=wl.LOSS_EXTERNAL_DY, seed=82)]
    inps = [wl.make_inputs(w, nonzero_state=True) for w in ws]
    want = [Session(w, i).run_and_fetch() for w, i in zip(ws, inps)]
    sessions = [Session(w, i) for w, i in zip(ws, inps)]
    streams = [torch.cuda.Stream() for _ in ws]
    torch.cuda.synchronize()
    errors, results = [], [[], []]

    def worker(k):
        try:
            for _ in range(5):
                sessions[k].run(stream=streams[k].cuda_stream)
                streams[k].synchronize()
                results[k].append(sessions[k].fetch())
        except Exception as exc:   # noqa: BLE001 - reported by the main thread
            errors.append(exc)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not errors, errors
    assert all(not th.is_alive() for th in threads)
    for k in range(2):
        assert len(results[k]) == 5
        for got in results[k]:
            _same(got, want[k])


def test_bounded_waits_give_up_and_report():
    """With the wait bound set to zero from the host, a workgroup that does not find the others'
    data at its first look gives up: every kernel still runs to its end, the run returns, the status
    word says a wait gave up and the session refuses the results.  With the default bound restored
    the same session computes the right gradients again."""
    from paper_1606_03401_amd.session import Session
    w = wl.Workload("give-up", B=64, I=128, H=128, t=60, kind=wl.KIND_HSM, m=60, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, seed=77)
    inp = wl.make_inputs(w)
    s = Session(w, inp)
    good = s.run_and_fetch()
    mb.mebptt_resident_wait_limit(0)
    try:
        with pytest.raises(RuntimeError):
            s.run_and_fetch()
        assert mb.mebptt_run_status(s.desc, s.workspace) == 1
    finally:
        mb.mebptt_resident_wait_limit(-1)
    _same(s.run_and_fetch(), good, "after restoring the bound")


@pytest.mark.parametrize("B,I,H,t", [(64, 128, 128, 40), (37, 100, 128, 33), (64, 256, 256, 50), (150, 128, 512, 30),
                                     (64, 256, 1024, 40)])
def test_gru_forward_chains(B, I, H, t):
    """The GRU core through forward-chain launches (h kept in full precision in registers from step
    to step), backward-only sweep launches and forward batches: bit for bit the launch-per-step
    path's gradients for every strategy and several budgets, and the oracle's within tolerance."""
    from paper_1606_03401_amd.session import Session
    from test_gpu_parity import TOL, check_against_oracle, oracle_gradients
    w = wl.Workload("gru-chain", B=B, I=I, H=H, t=t, kind=wl.KIND_HSM, m=4, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, dy_first_step=2, seed=1200 + B + H, cell=wl.CELL_GRU)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    base = _run(w, inp, wl.KIND_HSM, 3, chain=False)
    check_against_oracle(w, inp, base, oracle_gradients(w, inp), TOL[w.gemm_dtype], label=f"gru chain {B}x{I}x{H} per-step: ")
    for kind, m in ((wl.KIND_HSM, 1), (wl.KIND_HSM, 3), (wl.KIND_HSM, t), (wl.KIND_ISM, 2), (wl.KIND_ISM, t), (wl.KIND_MSM, 7)):
        _same(_run(w, inp, kind, m, chain=True), base, (kind, m))
    s = Session(w, inp, kind=wl.KIND_ISM, m=t)
    mb.mebptt_profile_enable(1)
    out = s.run_and_fetch()
    prof = mb.mebptt_profile_collect()
    mb.mebptt_profile_enable(0)
    _same(out, base, "profiled")
    assert prof.chain_steps >= t - 2 and prof.batch_steps == 0 and prof.sweep_forward_steps == 0
    assert mb.mebptt_run_status(s.desc, s.workspace) == 0
    assert prof.sweep_steps >= t - 40          # stored internal states: backward-only sweep launches
    s = Session(w, inp, kind=wl.KIND_HSM, m=t)
    mb.mebptt_profile_enable(1)
    out = s.run_and_fetch()
    prof = mb.mebptt_profile_collect()
    mb.mebptt_profile_enable(0)
    _same(out, base, "profiled, hidden states")
    assert prof.batch_steps >= t - 40 and prof.sweep_steps >= prof.batch_steps   # forward batches feed the sweeps


@pytest.mark.parametrize("B,I,H", [(64, 128, 128), (64, 256, 1024)])
def test_runs_join_the_chain_before_them(B, I, H):
    """Where memory runs out the schedule ends a re-forwarding chain with a run that leaves an internal
    state in the working core, then the backward operation on it, then the pairs for the steps below.
    That backward operation does not get a launch of its own: the sweep launch that follows carries
    it (recomputing the state itself and the chain stopping one step short, or taking the state from
    the core).  Counted from the launches, with every forward and backward operation still accounted
    for exactly once and the gradients those of the launch-per-step path bit for bit."""
    from paper_1606_03401_amd.session import Session
    t, m = 150, 7
    w = wl.Workload("join", B=B, I=I, H=H, t=t, kind=wl.KIND_HSM, m=m, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, seed=733 + H)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    base = _run(w, inp, wl.KIND_HSM, m, chain=False)
    s = Session(w, inp)
    sched = s.plan.schedule()
    CH = mb.mebptt_chunk_steps(s.desc)

    def pair_below(i):      # entries i, i + 1: forward operation of one step keeping its state, backward operation of it
        return (i + 1 < len(sched) and sched[i]["op"] == 1 and sched[i]["count"] == 1 and sched[i]["keep"]
                and sched[i + 1]["op"] == 2 and sched[i + 1]["step"] == sched[i]["step"])
    lone = [i for i in range(1, len(sched)) if sched[i]["op"] == 2 and sched[i - 1]["op"] == 1 and sched[i - 1]["count"] >= 2]
    joinable = [i for i in lone if pair_below(i + 1) and sched[i + 1]["step"] == sched[i]["step"] - 1
                and (sched[i]["step"] - 1) // CH == (sched[i]["step"] - 2) // CH]
    assert len(joinable) >= 10              # the schedule has many such backward operations ...
    lone, joinable = len(lone), len(joinable)
    mb.mebptt_profile_enable(1)
    out = s.run_and_fetch()
    prof = mb.mebptt_profile_collect()
    mb.mebptt_profile_enable(0)
    _same(out, base, "joined runs")
    assert mb.mebptt_run_status(s.desc, s.workspace) == 0
    # ... and none of them is launched alone (what is, are the ones no pair follows, and single pairs)
    assert prof.launches[mb.K_BACKWARD] + prof.launches[mb.K_PAIR] <= lone - joinable + 3
    assert (prof.launches[mb.K_FORWARD] + prof.launches[mb.K_PAIR] + prof.chain_steps + prof.sweep_forward_steps
            + prof.batch_steps == out.stats.forward_ops == s.plan.forward_ops)
    assert prof.launches[mb.K_BACKWARD] + prof.launches[mb.K_PAIR] + prof.sweep_steps == t


def test_batched_recomputation_with_the_loss_on_h():
    """The same path when the loss is half the sum of the squared outputs (dy_t = h_t): the backward-only
    sweep launch then takes the injected gradient from the states the forward-batch launch left in the
    stage."""
    from test_gpu_parity import TOL, check_against_oracle, oracle_gradients
    w = wl.Workload("batch-h2", B=64, I=64, H=1024, t=40, kind=wl.KIND_HSM, m=7, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_HALF_SUM_H2, seed=515)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    base = _run(w, inp, wl.KIND_HSM, 7, chain=False)
    for kind, m in ((wl.KIND_HSM, 7), (wl.KIND_HSM, 40), (wl.KIND_MSM, 25)):
        _same(_run(w, inp, kind, m, chain=True), base, (kind, m))
    check_against_oracle(w, inp, base, oracle_gradients(w, inp), TOL[w.gemm_dtype], label="batched recomputation, loss on h: ")


@pytest.mark.parametrize("B,I,H,t,m", [(64, 128, 128, 70, 6), (64, 256, 1024, 45, 8)])
def test_resident_launches_in_a_captured_graph(B, I, H, t, m):
    """A run whose sequential work goes out as chain, sweep and forward-batch launches, captured into
    a HIP graph: every replay -- with eager runs, clobbered outputs and synchronisations between
    them -- reproduces the eager result bit for bit and leaves the status word clear (the arrival
    counters the captured launches count on are cleared by the run's own first kernel)."""
    import torch
    from paper_1606_03401_amd.session import Session
    w = wl.Workload("graph-resident", B=B, I=I, H=H, t=t, kind=wl.KIND_HSM, m=m, gemm_dtype=wl.GEMM_BF16,
                    loss=wl.LOSS_EXTERNAL_DY, seed=610 + H)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    base = _run(w, inp, wl.KIND_HSM, m, chain=False)
    s = Session(w, inp)
    eager = s.run_and_fetch()
    _same(eager, base, "eager")
    s.capture()
    for rep in range(4):
        for tsr in (s.dW_ih, s.dW_hh, s.db, s.dh0, s.dc0, s.dx, s.y):
            tsr.fill_(float("nan"))
        torch.cuda.synchronize()
        s.replay()
        _same(s.fetch(), eager, ("replay", rep))
        assert mb.mebptt_run_status(s.desc, s.workspace) == 0
        if rep % 2 == 0:          # the program's own eager work between replays
            _same(s.run_and_fetch(), eager, ("eager after replay", rep))


def test_random_shapes_budgets_and_strategies_bit_identical():
    """Seeded random cases over the shape classes with resident launches, both cores, every strategy,
    budgets from 1 to beyond t, sequences from 2 steps to several chunks, losses starting anywhere:
    with the chain, sweep and forward-batch launches (and everything the executor does to join and
    lengthen them) the gradients are those of the launch-per-step path bit for bit and finite."""
    rng = np.random.default_rng(20260)
    for case in range(160):
        H = int(rng.choice([128, 256, 512, 1024]))
        I = {128: int(rng.choice([8, 40, 64, 100, 128])), 256: int(rng.choice([136, 200, 256])),
             512: int(rng.choice([16, 64, 100, 128])), 1024: int(rng.choice([32, 128, 250, 256]))}[H]
        B = int(rng.choice([1, 3, 8, 17, 32, 50, 64, 100, 128, 200, 256]))
        if H == 1024 and B > 128:
            B = 64
        t = int(rng.integers(2, 90)) if rng.random() < 0.85 else int(rng.integers(90, 300))
        kind = int(rng.choice([wl.KIND_HSM, wl.KIND_ISM, wl.KIND_MSM]))
        m = int(rng.integers(1, t + 2)) if kind != wl.KIND_MSM else int(rng.integers(2, 4 * t + 2))
        w = wl.Workload("random", B=B, I=I, H=H, t=t, kind=kind, m=m, gemm_dtype=wl.GEMM_BF16, loss=wl.LOSS_EXTERNAL_DY,
                        dy_first_step=int(rng.integers(1, t + 1)), seed=int(rng.integers(1, 10**6)),
                        cell=int(rng.random() < 0.2))
        inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
        what = (case, B, I, H, t, kind, m, w.dy_first_step, w.cell)
        base = _run(w, inp, kind, m, chain=False)
        got = _run(w, inp, kind, m, chain=True)
        _same(got, base, what)
        for f in FIELDS:
            assert np.all(np.isfinite(getattr(got, f))), (what, f)
