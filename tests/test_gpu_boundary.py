"""GPU tests of the boundary's memory and resource contract: the run stays inside the slot pool and
the workspace it was given and below the peak it reports (measured with guard bytes, not taken
from the plan); the two-call form (prepare + run_prepared) reproduces the one-call form bit for
bit; concurrent host threads are served; shutdown releases and the library works again."""
import threading

import numpy as np
import pytest

from paper_1606_03401_amd import binding as mb
from paper_1606_03401_amd import workloads as wl

pytestmark = pytest.mark.gpu

FIELDS = ("dW_ih", "dW_hh", "db", "dh0", "dc0", "dx", "y")
PATTERN = 0xA5
GUARD = 64 * 1024


def _same(a, b):
    for f in FIELDS:
        assert np.array_equal(getattr(a, f), getattr(b, f)), f


GUARD_SHAPES = [
    wl.Workload("guard-ragged", B=37, I=50, H=72, t=9, kind=wl.KIND_HSM, m=3, gemm_dtype=wl.GEMM_BF16,
                loss=wl.LOSS_EXTERNAL_DY, seed=41),
    wl.Workload("guard-ragged-gru", B=37, I=50, H=72, t=9, kind=wl.KIND_HSM, m=3, gemm_dtype=wl.GEMM_BF16,
                loss=wl.LOSS_EXTERNAL_DY, seed=42, cell=wl.CELL_GRU),
    wl.Workload("guard-multitile", B=130, I=100, H=1000, t=6, kind=wl.KIND_HSM, m=3, gemm_dtype=wl.GEMM_BF16,
                loss=wl.LOSS_EXTERNAL_DY, seed=43),
    wl.CONFIGS["cfg1"],
    wl.CONFIGS["cfg1"].scaled(gemm_dtype=wl.GEMM_BF16),
]


@pytest.mark.parametrize("w", GUARD_SHAPES, ids=lambda w: f"{w.name}-{'bf16' if w.gemm_dtype else 'f32'}")
def test_guard_bands_and_measured_peak(w):
    """Slot pool and workspace are interior, 256-byte aligned views of larger buffers filled with
    0xA5.  After a run of every strategy: the guard bytes on both sides of both buffers are
    untouched; no byte of the pool at or above the reported peak was written; the unit just below
    the peak was written (so the reported peak is the measured one); and the peak equals the
    plan's.  The pool is budgeted generously (m larger than needed for some cases) so that "above
    the peak" is not empty."""
    import torch
    from paper_1606_03401_amd.session import Session
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    base = None
    cases = [(wl.KIND_HSM, 1), (wl.KIND_HSM, 3), (wl.KIND_HSM, w.t + 4), (wl.KIND_ISM, 1), (wl.KIND_ISM, 2),
             (wl.KIND_ISM, w.t + 2), (wl.KIND_MSM, 2), (wl.KIND_MSM, 6), (wl.KIND_MSM, 4 * w.t + 5)]
    for kind, m in cases:
        s = Session(w, inp, kind=kind, m=m, guard_bytes=GUARD, fill_byte=PATTERN)
        assert s.slots.data_ptr() % 256 == 0 and s.workspace.data_ptr() % 256 == 0
        assert s.slots.data_ptr() == s.slots_outer.data_ptr() + GUARD
        out = s.run_and_fetch()
        torch.cuda.synchronize()
        for outer, inner_bytes, what in ((s.slots_outer, s.slot_bytes, "slot pool"), (s.workspace_outer, s.ws_bytes, "workspace")):
            lo, hi = outer[:GUARD], outer[GUARD + inner_bytes:]
            assert bool((lo == PATTERN).all()), f"{what}: bytes before the buffer were written ({kind}, {m})"
            assert bool((hi == PATTERN).all()), f"{what}: bytes after the buffer were written ({kind}, {m})"
        unit = mb.mebptt_unit_bytes(s.desc)
        per = 4 if kind == wl.KIND_ISM else 1
        assert out.stats.peak == s.plan.peak <= m
        assert out.stats.peak_slot_bytes <= out.stats.peak * per * unit <= s.slot_bytes
        high = out.stats.peak_slot_bytes
        assert high % unit == 0
        assert bool((s.slots[high:] == PATTERN).all()), f"pool written at or above the reported peak ({kind}, {m})"
        if high:
            assert not bool((s.slots[high - unit:high] == PATTERN).all()), f"top unit below the peak never written ({kind}, {m})"
        if base is None:
            base = out
        _same(out, base)
        del s


def test_prepare_then_run_matches_one_call():
    """mebptt_prepare + mebptt_run_prepared, several times on one workspace, with different plans
    and a shorter sequence in between (so a full chunk's staging precedes a short, padded one):
    every result is the one-call result bit for bit.  An unprepared workspace is refused."""
    from paper_1606_03401_amd.session import Session
    for w in (wl.Workload("prep", B=5, I=7, H=9, t=70, kind=wl.KIND_HSM, m=4, gemm_dtype=wl.GEMM_BF16,
                          loss=wl.LOSS_EXTERNAL_DY, seed=51),
              wl.Workload("prep32", B=37, I=50, H=72, t=40, kind=wl.KIND_MSM, m=9, gemm_dtype=wl.GEMM_FP32,
                          loss=wl.LOSS_EXTERNAL_DY, seed=52)):
        inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
        want = Session(w, inp).run_and_fetch()
        s = Session(w, inp)
        with pytest.raises(mb.MebpttError) as e:
            mb.mebptt_run_prepared(s.desc, s.plan, s.x, s.dy, s.h0, s.c0, s.slots, s.workspace, s.dW_ih, s.dW_hh, s.db,
                                   s.dh0, s.dc0)
        assert e.value.code == mb.EWORKSPACE
        s.prepare()
        _same(s.run_and_fetch(), want)
        _same(s.run_and_fetch(), want)            # staging left by the previous run
        # a shorter sequence on the same prepared workspace, then the long one again
        w2 = w.scaled(t=w.t - 27)
        inp2 = wl.Inputs(inp.W_ih, inp.W_hh, inp.b, inp.x[:w2.t], inp.dy[:w2.t], inp.h0, inp.c0)
        want2 = Session(w2, inp2).run_and_fetch()
        s2 = Session(w2, inp2)
        s2.workspace, s2.prepared = s.workspace, True
        _same(s2.run_and_fetch(), want2)
        _same(s.run_and_fetch(), want)
        _same(s2.run_and_fetch(), want2)


def test_two_host_threads():
    """Two host threads, each with its own stream, slot pool and workspace, call mebptt_run at the
    same time, repeatedly: the enqueue phases are serialised inside the library, and every result is
    the single-threaded one."""
    import torch
    from paper_1606_03401_amd.session import Session
    ws = [wl.Workload("thr-a", B=20, I=500, H=200, t=30, kind=wl.KIND_HSM, m=4, gemm_dtype=wl.GEMM_BF16,
                      loss=wl.LOSS_EXTERNAL_DY, seed=61),
          wl.Workload("thr-b", B=37, I=50, H=72, t=25, kind=wl.KIND_ISM, m=3, gemm_dtype=wl.GEMM_FP32,
                      loss=wl.LOSS_HALF_SUM_H2, seed=62)]
    inps = [wl.make_inputs(w, nonzero_state=True, nonzero_bias=True) for w in ws]
    want = [Session(w, i).run_and_fetch() for w, i in zip(ws, inps)]
    sessions = [Session(w, i) for w, i in zip(ws, inps)]
    streams = [torch.cuda.Stream() for _ in ws]
    torch.cuda.synchronize()
    errors, results = [], [[], []]

    def worker(k):
        try:
            for _ in range(6):
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
        assert len(results[k]) == 6
        for got in results[k]:
            _same(got, want[k])


def test_shutdown_and_reuse():
    from paper_1606_03401_amd.session import Session
    w = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(w)
    want = Session(w, inp).run_and_fetch()
    mb.mebptt_shutdown()
    mb.mebptt_shutdown()                     # nothing left to release: still fine
    _same(Session(w, inp).run_and_fetch(), want)
    us = mb.mebptt_null_launch_us(500)
    assert 0.2 < us < 100.0


def test_measurement_hooks():
    """The stand-alone measurements return sane values and leave the device usable: every
    synchronisation variant completes with status 0 (32 workgroups per XCD, no wait gave up, every
    exchanged word read back right), the per-XCD meeting is cheaper than the device-wide one, an
    event pair costs something but not much, and the chunk length follows the documented rule."""
    from paper_1606_03401_amd.session import Session
    us = []
    for variant in (0, 1, 2):
        t, status = mb.mebptt_measure_sync(variant, 500)
        assert status == 0, (variant, status)
        assert 0.05 < t < 100.0, (variant, t)
        us.append(t)
    assert us[1] < us[0]
    with pytest.raises(mb.MebpttError):
        mb.mebptt_measure_sync(3, 10)
    plain, bracketed = mb.mebptt_bracket_overhead_us(8.0, 50)
    assert 8.0 <= plain < 40.0 and plain < bracketed < plain + 40.0
    for name, ch in (("cfg2", 32), ("cfg3", 32), ("cfg5", 64), ("cfg1", 64)):
        w = wl.CONFIGS[name]
        desc = mb.make_desc(w.B, w.I, w.H, w.t, w.gemm_dtype, w.loss, w.dy_first_step)
        assert mb.mebptt_chunk_steps(desc) == ch
    w = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(w)
    a = Session(w, inp).run_and_fetch()
    _same(Session(w, inp).run_and_fetch(), a)
