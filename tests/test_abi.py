"""The C-ABI library loads without a GPU and exports every function `include/mebptt.h` declares;
the size queries (pure host arithmetic) behave."""
import ctypes
import os
import re

from paper_1606_03401_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mebptt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(mebptt_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared_functions()
    assert "mebptt_plan" in names and "mebptt_run" in names and len(names) >= 18
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_1606_03401_amd", "libmebptt.so"))
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
        assert n in mb.SIGNATURES, f"{n} has no binding"
    assert set(mb.SIGNATURES) == set(names)
    assert "gfx950" in mb.mebptt_version()


def test_recomputation_stage_in_the_workspace():
    """The workspace carries a stage for recomputed internal states exactly on the shapes whose way
    back through stored hidden states is a forward-batch launch plus a backward-only sweep launch:
    bf16 operands, a shape the backward-only sweep kernel covers, and no sweep launch that recomputes
    internal states itself (the LSTM has those up to H = 512; the GRU has none).  As many states as
    a sweep launch carries (32), at most 48 MiB, three units each."""
    def desc(B, I, H, cell=0, dtype=1):
        return mb.make_desc(B, I, H, 100, dtype, 0, 1, cell)
    unit = lambda B, H: mb.mebptt_unit_bytes(desc(B, 64, H))
    assert mb.mebptt_stage_steps(desc(64, 256, 1024)) == 32 and 32 * 3 * unit(64, 1024) == 48 << 20
    assert mb.mebptt_stage_steps(desc(128, 64, 1024)) == 16 and 16 * 3 * unit(128, 1024) == 48 << 20
    for B, I, H in ((256, 128, 512), (64, 256, 256), (64, 128, 128)):      # the sweep launch recomputes the states itself
        assert mb.mebptt_stage_steps(desc(B, I, H)) == 0
        assert mb.mebptt_stage_steps(desc(B, I, H, cell=1)) > 0           # the GRU has no such launch
    for B, I, H in ((128, 512, 2048), (200, 64, 1024), (32, 1024, 4096)):  # no backward-only sweep launch for the shape
        assert mb.mebptt_stage_steps(desc(B, I, H)) == 0 and mb.mebptt_stage_steps(desc(B, I, H, cell=1)) == 0
    assert mb.mebptt_stage_steps(desc(64, 256, 1024, dtype=0)) == 0       # fp32 operands: launch-per-step kernels only
    # the stage is part of the workspace, which does not depend on t
    with_stage, without = desc(64, 256, 1024), desc(64, 256, 1024, dtype=0)
    assert mb.mebptt_workspace_bytes(with_stage) == mb.mebptt_workspace_bytes(mb.make_desc(64, 256, 1024, 5, 1, 0, 1, 0))
    assert mb.mebptt_workspace_bytes(with_stage) > 48 << 20 and without is not None


def test_size_queries():
    d = mb.make_desc(64, 256, 1024, 1000, 1, 0, 1)
    unit = 2 * 64 * 1024 * 4
    assert mb.mebptt_unit_bytes(d) == unit
    p = mb.mebptt_plan(1000, 50, mb.HSM)
    assert mb.mebptt_slot_pool_bytes(d, p) == 50 * unit
    p = mb.mebptt_plan(1000, 100, mb.ISM)
    assert mb.mebptt_slot_pool_bytes(d, p) == 100 * 4 * unit
    ws = mb.mebptt_workspace_bytes(d)
    assert 0 < ws < 192 << 20          # operand copies, chunk buffers of the batched GEMMs, recomputation stage (<= 48 MiB)
    # independent of t
    assert mb.mebptt_workspace_bytes(mb.make_desc(64, 256, 1024, 7, 1, 0, 1)) == ws
    assert mb.mebptt_units_for_bytes(d, mb.MSM, 4_000_000_000) == 4_000_000_000 // unit
    assert mb.mebptt_units_for_bytes(d, mb.ISM, 4_000_000_000) == 4_000_000_000 // (4 * unit)
    assert mb.mebptt_units_for_bytes(d, mb.HSM, unit - 1) == 0
    assert mb.mebptt_workspace_bytes(mb.make_desc(0, 256, 1024, 7, 1, 0, 1)) == 0
