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
    back through stored hidden states is a forward-batch launch plus a backward-only sweep launch
    (bf16 LSTM, H = 1024, a batch the sweep kernel covers): as many states as a sweep launch carries
    (32), at most 48 MiB, three units each.  The GRU of the same shape has the same workspace but for
    the stage."""
    def ws(B, I, H, cell):
        return mb.mebptt_workspace_bytes(mb.make_desc(B, I, H, 100, 1, 0, 1, cell))
    unit = lambda B, H: mb.mebptt_unit_bytes(mb.make_desc(B, 64, H, 100, 1, 0, 1, 0))
    assert ws(64, 256, 1024, 0) - ws(64, 256, 1024, 1) == 32 * 3 * unit(64, 1024) == 48 << 20
    assert ws(128, 64, 1024, 0) - ws(128, 64, 1024, 1) == 16 * 3 * unit(128, 1024) == 48 << 20
    for B, I, H in ((256, 128, 512), (128, 512, 2048), (200, 64, 1024), (64, 256, 256)):
        assert ws(B, I, H, 0) == ws(B, I, H, 1), (B, I, H)      # no stage: sweeps with forward operations, or no sweeps
    assert ws(64, 256, 1024, 0) == mb.mebptt_workspace_bytes(mb.make_desc(64, 256, 1024, 5, 1, 0, 1, 0))   # independent of t


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
