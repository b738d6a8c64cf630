"""GPU test of mebptt_run_static, the entry point for callers that cannot allocate: through the C
ABI, against mebptt_run on the same inputs, bit for bit, on two calls in a row -- the second with a
smaller input, so that it runs on whatever the first left in the shared static array -- and the
refusal of a shape whose workspace exceeds the array."""
import numpy as np
import pytest

from paper_1606_03401_amd import binding as mb
from paper_1606_03401_amd import workloads as wl

pytestmark = pytest.mark.gpu

FIELDS = ("dW_ih", "dW_hh", "db", "dh0", "dc0", "dx", "y")


def _pair(w, kind, m):
    from paper_1606_03401_amd.session import Session
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    want = Session(w, inp, kind=kind, m=m).run_and_fetch()
    s = Session(w, inp, kind=kind, m=m, static_workspace=True)
    assert s.ws_bytes <= mb.mebptt_static_workspace_bytes()
    got = s.run_and_fetch()
    assert got.stats.forward_ops == want.stats.forward_ops and got.stats.backward_ops == w.t
    assert got.stats.peak == want.stats.peak
    for f in FIELDS:
        assert np.array_equal(getattr(got, f), getattr(want, f)), (w.name, kind, m, f)
    return s, inp, want


def test_static_workspace_matches_mebptt_run_twice_in_a_row():
    big = wl.Workload("static-big", B=37, I=50, H=72, t=41, kind=wl.KIND_MSM, m=9, gemm_dtype=wl.GEMM_BF16,
                      loss=wl.LOSS_EXTERNAL_DY, seed=71)
    small = wl.Workload("static-small", B=5, I=7, H=9, t=6, kind=wl.KIND_HSM, m=3, gemm_dtype=wl.GEMM_BF16,
                        loss=wl.LOSS_EXTERNAL_DY, seed=72)
    _pair(big, wl.KIND_MSM, 9)
    _pair(small, wl.KIND_HSM, 3)          # smaller input on the array the first call used
    _pair(wl.CONFIGS["cfg1"], wl.KIND_ISM, 2)   # fp32 operands after bf16 ones
    s, inp, want = _pair(big, wl.KIND_HSM, 2)
    again = s.run_and_fetch()             # the same session twice
    for f in FIELDS:
        assert np.array_equal(getattr(again, f), getattr(want, f)), f


def test_static_workspace_refuses_large_shapes():
    import torch
    from paper_1606_03401_amd.session import Session
    w = wl.CONFIGS["cfg2"].scaled(t=4, m=2)
    inp = wl.make_inputs(w)
    s = Session(w, inp, static_workspace=True)
    assert s.ws_bytes > mb.mebptt_static_workspace_bytes()
    s.dW_ih.fill_(7.0)
    with pytest.raises(mb.MebpttError) as e:
        s.run()
    assert e.value.code == mb.EWORKSPACE
    torch.cuda.synchronize()
    assert bool((s.dW_ih == 7.0).all())
