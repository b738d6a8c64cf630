"""Buffer management around ``mebptt_run`` for tests and benchmarks.

Allocates the device buffers a run needs through PyTorch (inputs, outputs, slot pool,
workspace) and calls the binding.  It performs no arithmetic of its own.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
import torch

from . import binding as mb
from .workloads import Inputs, Workload


@dataclasses.dataclass
class Outputs:
    dW_ih: np.ndarray
    dW_hh: np.ndarray
    db: np.ndarray
    dh0: np.ndarray
    dc0: np.ndarray
    dx: Optional[np.ndarray]
    y: Optional[np.ndarray]
    stats: mb.mebptt_stats


class Session:
    """Device-resident inputs and outputs of one workload; `run` enqueues one gradient step."""

    def __init__(self, w: Workload, inp: Inputs, *, kind: Optional[int] = None, m: Optional[int] = None,
                 gemm_dtype: Optional[int] = None, want_dx: bool = True, want_y: bool = True,
                 pass_null_state: bool = False, device: str = "cuda:0", plan: Optional[mb.Plan] = None,
                 guard_bytes: int = 0, fill_byte: int = 0xFF, static_workspace: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("mebptt needs a GPU: no HIP device is visible")
        self.w = w
        self.dev = torch.device(device)
        self.kind = w.kind if kind is None else kind
        self.m = w.m if m is None else m
        self.desc = mb.make_desc(w.B, w.I, w.H, w.t, w.gemm_dtype if gemm_dtype is None else gemm_dtype, w.loss,
                                 w.dy_first_step, w.cell)
        self.plan = plan if plan is not None else mb.mebptt_plan(w.t, self.m, self.kind, w.alpha, w.beta)
        dev = self.dev
        up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.W_ih, self.W_hh, self.b, self.x, self.dy = up(inp.W_ih), up(inp.W_hh), up(inp.b), up(inp.x), up(inp.dy)
        self.h0 = None if pass_null_state else up(inp.h0)
        self.c0 = None if pass_null_state else up(inp.c0)
        f32 = dict(dtype=torch.float32, device=dev)
        gates, biases = (3, 6) if w.cell == mb.CELL_GRU else (4, 4)
        self.dW_ih = torch.empty((gates * w.H, w.I), **f32)
        self.dW_hh = torch.empty((gates * w.H, w.H), **f32)
        self.db = torch.empty((biases * w.H,), **f32)
        self.dh0 = torch.empty((w.B, w.H), **f32)
        self.dc0 = torch.empty((w.B, w.H), **f32)
        self.dx = torch.empty((w.t, w.B, w.I), **f32) if want_dx else None
        self.y = torch.empty((w.t, w.B, w.H), **f32) if want_y else None
        self.slot_bytes = mb.mebptt_slot_pool_bytes(self.desc, self.plan)
        self.ws_bytes = mb.mebptt_workspace_bytes(self.desc)
        # 0xFF bytes are NaNs as float32: stale memory can never pass for a valid result.  With
        # guard_bytes > 0 (a multiple of 256) the pool and the workspace are interior views of larger
        # buffers filled with the same byte, so that a test can see any write outside them.
        if guard_bytes % 256:
            raise ValueError("guard_bytes must be a multiple of 256")
        self.guard_bytes, self.fill_byte = guard_bytes, fill_byte
        self.slots_outer = torch.full((self.slot_bytes + 2 * guard_bytes,), fill_byte, dtype=torch.uint8, device=dev)
        self.slots = self.slots_outer[guard_bytes:guard_bytes + self.slot_bytes]
        self.static_workspace = static_workspace
        if static_workspace:
            self.workspace_outer = self.workspace = None
        else:
            self.workspace_outer = torch.full((self.ws_bytes + 2 * guard_bytes,), fill_byte, dtype=torch.uint8, device=dev)
            self.workspace = self.workspace_outer[guard_bytes:guard_bytes + self.ws_bytes]
        self.prepared = False

    def run(self, stream: Optional[int] = None) -> mb.mebptt_stats:
        if self.static_workspace:
            return mb.mebptt_run_static(self.desc, self.plan, self.W_ih, self.W_hh, self.b, self.x, self.dy, self.h0,
                                        self.c0, self.slots, self.dW_ih, self.dW_hh, self.db, self.dh0, self.dc0,
                                        self.dx, self.y, stream)
        if self.prepared:
            return mb.mebptt_run_prepared(self.desc, self.plan, self.x, self.dy, self.h0, self.c0, self.slots,
                                          self.workspace, self.dW_ih, self.dW_hh, self.db, self.dh0, self.dc0,
                                          self.dx, self.y, stream)
        return mb.mebptt_run(self.desc, self.plan, self.W_ih, self.W_hh, self.b, self.x, self.dy, self.h0, self.c0,
                             self.slots, self.workspace, self.dW_ih, self.dW_hh, self.db, self.dh0, self.dc0,
                             self.dx, self.y, stream)

    def prepare(self, stream: Optional[int] = None) -> None:
        """Builds the operand copies of the weights once; later `run` calls skip that work."""
        mb.mebptt_prepare(self.desc, self.W_ih, self.W_hh, self.b, self.workspace, stream)
        self.prepared = True

    def capture(self) -> None:
        """Records one gradient step into a HIP graph (the schedule and every pointer are fixed, so
        the run is a static sequence of kernel launches); `replay` then re-issues it without the
        per-launch host cost.  One eager run comes first so that nothing is created under capture."""
        self.run()
        torch.cuda.synchronize(self.dev)
        self._graph_stream = torch.cuda.Stream(device=self.dev)
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph, stream=self._graph_stream):
            self._graph_stats = self.run(stream=self._graph_stream.cuda_stream)

    def replay(self) -> None:
        self._graph.replay()

    def check_status(self) -> None:
        """Raises if a launch of the last run gave up (see mebptt_run_status)."""
        if self.workspace is None:
            return
        status = mb.mebptt_run_status(self.desc, self.workspace)
        if status:
            raise RuntimeError(f"mebptt run gave up with status {status}: outputs are invalid")

    def fetch(self, stats=None) -> Outputs:
        torch.cuda.synchronize(self.dev)
        self.check_status()
        dn = lambda t: None if t is None else t.cpu().numpy()
        return Outputs(dn(self.dW_ih), dn(self.dW_hh), dn(self.db), dn(self.dh0), dn(self.dc0), dn(self.dx),
                       dn(self.y), stats)

    def run_and_fetch(self) -> Outputs:
        stats = self.run()
        torch.cuda.synchronize(self.dev)
        self.check_status()
        dn = lambda t: None if t is None else t.cpu().numpy()
        return Outputs(dn(self.dW_ih), dn(self.dW_hh), dn(self.db), dn(self.dh0), dn(self.dc0), dn(self.dx),
                       dn(self.y), stats)
