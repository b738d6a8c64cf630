"""ctypes binding of ``libmebptt.so`` -- argument marshalling only.

Every function here has the name of the C entry point it calls (see ``include/mebptt.h``); all
planning and all arithmetic run inside the library.  PyTorch appears only as the owner of
device memory and of the HIP stream.  There is no fallback: if the library has not been built
the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmebptt.so")
_lib = None

OK, EINVAL, ENOMEM_SLOTS, EWORKSPACE, ESHAPE, EINFEASIBLE, EHIP, ENOMEM_HOST = 0, -1, -2, -3, -4, -5, -6, -7
HSM, ISM, MSM = 0, 1, 2
OP_FWD_RUN, OP_BWD = 1, 2
LOC_NONE, LOC_T0, LOC_T1, LOC_CORE, LOC_INIT = -1, -2, -3, -4, -5
COST_INF = 1 << 60


class MebpttError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"mebptt error {code}: {message}")
        self.code = code


class mebptt_op(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "step", "count", "src", "dst", "keep", "prev")]


class mebptt_decision(C.Structure):
    _fields_ = [("store", C.c_int32), ("y", C.c_int32)]


STORE_HIDDEN, STORE_INTERNAL = 1, 2


class mebptt_layer(C.Structure):
    _fields_ = [("cost", C.c_int64), ("state_units", C.c_int32), ("work_units", C.c_int32)]


class mebptt_chain_op(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "layer", "count", "src", "dst")]


class mebptt_chain_desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("B", C.c_int32), ("widths", C.POINTER(C.c_int32)), ("unit_bytes", C.c_size_t)]


class mebptt_chain_stats(C.Structure):
    _fields_ = [("forward_cost", C.c_int64), ("backward_ops", C.c_int64), ("peak_units", C.c_int32),
                ("reserved", C.c_int32)]


CHAIN_FORWARD, CHAIN_BACKWARD = 1, 2
CHAIN_INPUT, CHAIN_WORKING = -1, -2


class mebptt_lstm_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "I", "H", "t", "gemm_dtype", "loss", "dy_first_step", "cell")]


CELL_LSTM, CELL_GRU = 0, 1


class mebptt_stats(C.Structure):
    _fields_ = [("forward_ops", C.c_int64), ("backward_ops", C.c_int64), ("peak", C.c_int32),
                ("reserved", C.c_int32), ("peak_slot_bytes", C.c_size_t)]


K_FORWARD, K_BACKWARD, K_WGRAD, K_DGRAD, K_SETUP, K_PAIR, K_CHAIN, K_SWEEP, K_FWD_BATCH, K_CLASSES = 0, 1, 2, 3, 4, 5, 6, 7, 8, 9
K_NAMES = ("forward", "backward", "wgrad", "dgrad", "setup", "backward+forward", "forward chain", "sweep",
           "forward batch")


class mebptt_profile(C.Structure):
    _fields_ = [("launches", C.c_int64 * K_CLASSES), ("sampled", C.c_int64 * K_CLASSES),
                ("sampled_ms", C.c_double * K_CLASSES), ("forward_run_launches", C.c_int64),
                ("forward_run_ms", C.c_double), ("chain_steps", C.c_int64), ("chain_ms", C.c_double),
                ("sweep_steps", C.c_int64), ("sweep_ms", C.c_double), ("sampled_groups", C.c_int64 * K_CLASSES),
                ("sweep_forward_steps", C.c_int64), ("batch_steps", C.c_int64), ("batch_ms", C.c_double)]


# name -> (restype, argtypes): every symbol the header declares
_P = C.c_void_p
_DESC = C.POINTER(mebptt_lstm_desc)
SIGNATURES = {
    "mebptt_plan": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(_P)]),
    "mebptt_plan_from_policy": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(mebptt_decision),
                                          C.c_size_t, C.POINTER(_P)]),
    "mebptt_plan_chen_sqrt": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.POINTER(_P)]),
    "mebptt_plan_chen_recursive": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(_P)]),
    "mebptt_plan_free": (None, [_P]),
    "mebptt_chain_plan": (C.c_int, [C.POINTER(mebptt_layer), C.c_int32, C.c_int32, C.POINTER(_P)]),
    "mebptt_chain_plan_free": (None, [_P]),
    "mebptt_chain_cost": (C.c_int64, [_P, C.c_int32, C.c_int32, C.c_int32]),
    "mebptt_chain_split": (C.c_int32, [_P, C.c_int32, C.c_int32, C.c_int32]),
    "mebptt_chain_plan_forward_cost": (C.c_int64, [_P]),
    "mebptt_chain_plan_peak": (C.c_int32, [_P]),
    "mebptt_chain_plan_schedule": (C.POINTER(mebptt_chain_op), [_P, C.POINTER(C.c_size_t)]),
    "mebptt_chain_plan_layers": (C.POINTER(mebptt_layer), [_P, C.POINTER(C.c_int32)]),
    "mebptt_chain_layers": (C.c_int, [C.POINTER(mebptt_chain_desc), C.POINTER(mebptt_layer)]),
    "mebptt_chain_workspace_bytes": (C.c_size_t, [C.POINTER(mebptt_chain_desc)]),
    "mebptt_chain_run": (C.c_int, [C.POINTER(mebptt_chain_desc), _P, C.POINTER(_P), C.POINTER(_P), _P, _P, _P, C.c_size_t,
                                   _P, C.c_size_t, C.POINTER(_P), C.POINTER(_P), _P, _P, C.POINTER(mebptt_chain_stats), _P]),
    "mebptt_plan_cost": (C.POINTER(C.c_int64), [_P, C.c_int32]),
    "mebptt_plan_split": (C.POINTER(C.c_int32), [_P, C.c_int32]),
    "mebptt_plan_choice": (C.POINTER(C.c_uint8), [_P]),
    "mebptt_plan_length": (C.c_int32, [_P]),
    "mebptt_plan_budget": (C.c_int32, [_P]),
    "mebptt_plan_kind": (C.c_int32, [_P]),
    "mebptt_plan_forward_ops": (C.c_int64, [_P]),
    "mebptt_plan_peak": (C.c_int32, [_P]),
    "mebptt_plan_schedule": (C.POINTER(mebptt_op), [_P, C.POINTER(C.c_size_t)]),
    "mebptt_unit_bytes": (C.c_size_t, [_DESC]),
    "mebptt_slot_pool_bytes": (C.c_size_t, [_DESC, _P]),
    "mebptt_workspace_bytes": (C.c_size_t, [_DESC]),
    "mebptt_units_for_bytes": (C.c_int32, [_DESC, C.c_int32, C.c_size_t]),
    "mebptt_run": (C.c_int, [_DESC, _P] + [_P] * 7 + [_P, C.c_size_t, _P, C.c_size_t] + [_P] * 7
                   + [C.POINTER(mebptt_stats), _P]),
    "mebptt_prepare": (C.c_int, [_DESC] + [_P] * 3 + [_P, C.c_size_t, _P]),
    "mebptt_run_prepared": (C.c_int, [_DESC, _P] + [_P] * 4 + [_P, C.c_size_t, _P, C.c_size_t] + [_P] * 7
                            + [C.POINTER(mebptt_stats), _P]),
    "mebptt_run_static": (C.c_int, [_DESC, _P] + [_P] * 7 + [_P, C.c_size_t] + [_P] * 7
                          + [C.POINTER(mebptt_stats), _P]),
    "mebptt_static_workspace_bytes": (C.c_size_t, []),
    "mebptt_run_status": (C.c_int, [_DESC, _P, C.c_size_t, _P, C.POINTER(C.c_int32)]),
    "mebptt_forward_chain_enable": (C.c_int, [C.c_int32]),
    "mebptt_resident_wait_limit": (C.c_int, [C.c_int64]),
    "mebptt_shutdown": (C.c_int, []),
    "mebptt_null_launch_us": (C.c_int, [C.c_int32, _P, C.POINTER(C.c_double)]),
    "mebptt_measure_sync": (C.c_int, [C.c_int32, C.c_int32, _P, C.POINTER(C.c_double), C.POINTER(C.c_int32)]),
    "mebptt_chunk_steps": (C.c_int32, [_DESC]),
    "mebptt_stage_steps": (C.c_int32, [_DESC]),
    "mebptt_measure_forward_stream": (C.c_int, [_DESC, _P, C.c_size_t, C.c_int32, _P, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "mebptt_bracket_overhead_us": (C.c_int, [C.c_double, C.c_int32, _P, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "mebptt_measure_gemms": (C.c_int, [_DESC, _P, C.c_size_t, C.c_int32, _P, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "mebptt_profile_enable": (C.c_int, [C.c_int32]),
    "mebptt_profile_collect": (C.c_int, [C.POINTER(mebptt_profile)]),
    "mebptt_last_error": (C.c_char_p, []),
    "mebptt_version": (C.c_char_p, []),
}


def lib() -> C.CDLL:
    """Loads the library on first use.  Raises if it is missing: there is no other code path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_1606_03401_amd.build`")
        l = C.CDLL(_LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def mebptt_last_error() -> str:
    return lib().mebptt_last_error().decode()


def mebptt_version() -> str:
    return lib().mebptt_version().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise MebpttError(rc, mebptt_last_error())


class Plan:
    """Owner of a ``mebptt_plan_t*``; the table properties are read-only numpy views of the
    library's memory (valid while this object lives)."""

    def __init__(self, handle: int):
        self.handle = handle

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.mebptt_plan_free(self.handle)
            self.handle = None

    @property
    def t(self) -> int:
        return lib().mebptt_plan_length(self.handle)

    @property
    def m(self) -> int:
        return lib().mebptt_plan_budget(self.handle)

    @property
    def kind(self) -> int:
        return lib().mebptt_plan_kind(self.handle)

    @property
    def forward_ops(self) -> int:
        return lib().mebptt_plan_forward_ops(self.handle)

    @property
    def peak(self) -> int:
        return lib().mebptt_plan_peak(self.handle)

    def _table(self, ptr, dtype):
        if not ptr:
            return None
        shape = (self.t + 1, self.m + 1)
        a = np.ctypeslib.as_array(ptr, shape=shape)
        a = a.view(dtype)
        a.flags.writeable = False
        return a

    def cost(self, which: int = 0):
        return self._table(lib().mebptt_plan_cost(self.handle, which), np.int64)

    def split(self, which: int = 0):
        return self._table(lib().mebptt_plan_split(self.handle, which), np.int32)

    def choice(self):
        return self._table(lib().mebptt_plan_choice(self.handle), np.uint8)

    def schedule(self) -> np.ndarray:
        """Structured array with fields op, step, count, src, dst, keep, prev (a copy)."""
        n = C.c_size_t(0)
        ptr = lib().mebptt_plan_schedule(self.handle, C.byref(n))
        dt = np.dtype([(f, np.int32) for f, _ in mebptt_op._fields_])
        if n.value == 0:
            return np.zeros(0, dt)
        raw = np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_int32)), shape=(n.value, 7))
        return raw.copy().view(dt).reshape(n.value)


def mebptt_plan(t: int, m: int, kind: int, alpha: int = 4, beta: int = 3) -> Plan:
    out = _P()
    _check(lib().mebptt_plan(t, m, kind, alpha, beta, C.byref(out)))
    return Plan(out.value)


class ChainPlan:
    """Owner of a ``mebptt_chain_plan_t*`` (non-homogeneous chain; planning only)."""

    def __init__(self, handle: int, n: int, m: int):
        self.handle, self.n, self.m = handle, n, m

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.mebptt_chain_plan_free(self.handle)
            self.handle = None

    def cost(self, t: int, m: int, x: int) -> int:
        return lib().mebptt_chain_cost(self.handle, t, m, x)

    def split(self, t: int, m: int, x: int) -> int:
        return lib().mebptt_chain_split(self.handle, t, m, x)

    @property
    def forward_cost(self) -> int:
        return lib().mebptt_chain_plan_forward_cost(self.handle)

    @property
    def peak(self) -> int:
        return lib().mebptt_chain_plan_peak(self.handle)

    def schedule(self) -> np.ndarray:
        n = C.c_size_t(0)
        ptr = lib().mebptt_chain_plan_schedule(self.handle, C.byref(n))
        dt = np.dtype([(f, np.int32) for f, _ in mebptt_chain_op._fields_])
        if n.value == 0:
            return np.zeros(0, dt)
        raw = np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_int32)), shape=(n.value, 5))
        return raw.copy().view(dt).reshape(n.value)


def mebptt_chain_plan(layers, m: int) -> ChainPlan:
    """`layers`: sequence of (cost, state_units, work_units)."""
    arr = (mebptt_layer * max(len(layers), 1))(*[mebptt_layer(int(u), int(s), int(p)) for u, s, p in layers])
    out = _P()
    _check(lib().mebptt_chain_plan(arr, len(layers), m, C.byref(out)))
    return ChainPlan(out.value, len(layers), m)


def mebptt_plan_from_policy(t: int, m: int, decisions, alpha: int = 4, beta: int = 3) -> Plan:
    """`decisions`: sequence of (store, y) pairs, store = STORE_HIDDEN or STORE_INTERNAL."""
    arr = (mebptt_decision * max(len(decisions), 1))(*[mebptt_decision(int(s), int(y)) for s, y in decisions])
    out = _P()
    _check(lib().mebptt_plan_from_policy(t, m, alpha, beta, arr, len(decisions), C.byref(out)))
    return Plan(out.value)


def mebptt_plan_chen_sqrt(t: int, alpha: int = 4, beta: int = 3) -> Plan:
    out = _P()
    _check(lib().mebptt_plan_chen_sqrt(t, alpha, beta, C.byref(out)))
    return Plan(out.value)


def mebptt_plan_chen_recursive(t: int, k: int, alpha: int = 4, beta: int = 3) -> Plan:
    out = _P()
    _check(lib().mebptt_plan_chen_recursive(t, k, alpha, beta, C.byref(out)))
    return Plan(out.value)


def make_desc(B: int, I: int, H: int, t: int, gemm_dtype: int, loss: int, dy_first_step: int = 1,
              cell: int = CELL_LSTM) -> mebptt_lstm_desc:
    return mebptt_lstm_desc(B, I, H, t, gemm_dtype, loss, dy_first_step, cell)


def mebptt_unit_bytes(desc: mebptt_lstm_desc) -> int:
    return lib().mebptt_unit_bytes(C.byref(desc))


def mebptt_slot_pool_bytes(desc: mebptt_lstm_desc, plan: Plan) -> int:
    return lib().mebptt_slot_pool_bytes(C.byref(desc), plan.handle)


def mebptt_workspace_bytes(desc: mebptt_lstm_desc) -> int:
    return lib().mebptt_workspace_bytes(C.byref(desc))


def mebptt_units_for_bytes(desc: mebptt_lstm_desc, kind: int, budget_bytes: int) -> int:
    return lib().mebptt_units_for_bytes(C.byref(desc), kind, budget_bytes)


def mebptt_profile_enable(every_n: int) -> None:
    _check(lib().mebptt_profile_enable(every_n))


def mebptt_profile_collect() -> mebptt_profile:
    out = mebptt_profile()
    _check(lib().mebptt_profile_collect(C.byref(out)))
    return out


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to mebptt_run must be contiguous")
    return t.data_ptr()


def mebptt_run(desc: mebptt_lstm_desc, plan: Plan, W_ih, W_hh, b, x, dy, h0, c0, slots, workspace,
               dW_ih, dW_hh, db, dh0, dc0, dx=None, y_out=None, stream: Optional[int] = None) -> mebptt_stats:
    """Enqueues one gradient step.  Tensor arguments are torch CUDA tensors (float32; `slots` and
    `workspace` are uint8 buffers); `stream` is a raw hipStream_t (default: torch's current stream).
    Returns the host-side statistics.  The caller synchronises."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    stats = mebptt_stats()
    rc = lib().mebptt_run(C.byref(desc), plan.handle, _ptr(W_ih), _ptr(W_hh), _ptr(b), _ptr(x), _ptr(dy), _ptr(h0),
                          _ptr(c0), _ptr(slots), slots.numel() * slots.element_size(), _ptr(workspace),
                          workspace.numel() * workspace.element_size(), _ptr(dW_ih), _ptr(dW_hh), _ptr(db), _ptr(dh0),
                          _ptr(dc0), _ptr(dx), _ptr(y_out), C.byref(stats), stream)
    _check(rc)
    return stats


def _stream(stream: Optional[int]) -> int:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return stream


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def mebptt_prepare(desc: mebptt_lstm_desc, W_ih, W_hh, b, workspace, stream: Optional[int] = None) -> None:
    """Builds the operand copies of the weights inside `workspace` (see mebptt_run_prepared)."""
    _check(lib().mebptt_prepare(C.byref(desc), _ptr(W_ih), _ptr(W_hh), _ptr(b), _ptr(workspace), _nbytes(workspace),
                                _stream(stream)))


def mebptt_run_prepared(desc: mebptt_lstm_desc, plan: Plan, x, dy, h0, c0, slots, workspace, dW_ih, dW_hh, db, dh0,
                        dc0, dx=None, y_out=None, stream: Optional[int] = None) -> mebptt_stats:
    """mebptt_run on a workspace that mebptt_prepare has filled for these weights."""
    stats = mebptt_stats()
    _check(lib().mebptt_run_prepared(C.byref(desc), plan.handle, _ptr(x), _ptr(dy), _ptr(h0), _ptr(c0), _ptr(slots),
                                     _nbytes(slots), _ptr(workspace), _nbytes(workspace), _ptr(dW_ih), _ptr(dW_hh),
                                     _ptr(db), _ptr(dh0), _ptr(dc0), _ptr(dx), _ptr(y_out), C.byref(stats),
                                     _stream(stream)))
    return stats


def mebptt_run_static(desc: mebptt_lstm_desc, plan: Plan, W_ih, W_hh, b, x, dy, h0, c0, slots, dW_ih, dW_hh, db, dh0,
                      dc0, dx=None, y_out=None, stream: Optional[int] = None) -> mebptt_stats:
    """mebptt_run with the workspace in the library's static device array: allocates nothing."""
    stats = mebptt_stats()
    _check(lib().mebptt_run_static(C.byref(desc), plan.handle, _ptr(W_ih), _ptr(W_hh), _ptr(b), _ptr(x), _ptr(dy),
                                   _ptr(h0), _ptr(c0), _ptr(slots), _nbytes(slots), _ptr(dW_ih), _ptr(dW_hh), _ptr(db),
                                   _ptr(dh0), _ptr(dc0), _ptr(dx), _ptr(y_out), C.byref(stats), _stream(stream)))
    return stats


def mebptt_static_workspace_bytes() -> int:
    return lib().mebptt_static_workspace_bytes()


def mebptt_run_status(desc: mebptt_lstm_desc, workspace, stream: Optional[int] = None) -> int:
    """Waits for the stream and returns the status word of the last run on `workspace` (0 = fine)."""
    out = C.c_int32(0)
    _check(lib().mebptt_run_status(C.byref(desc), _ptr(workspace), _nbytes(workspace), _stream(stream), C.byref(out)))
    return out.value


def mebptt_forward_chain_enable(on: bool) -> None:
    _check(lib().mebptt_forward_chain_enable(1 if on else 0))


def mebptt_resident_wait_limit(ticks: int) -> None:
    _check(lib().mebptt_resident_wait_limit(int(ticks)))


def mebptt_shutdown() -> None:
    _check(lib().mebptt_shutdown())


def mebptt_null_launch_us(launches: int = 2000, stream: Optional[int] = None) -> float:
    out = C.c_double(0.0)
    _check(lib().mebptt_null_launch_us(launches, _stream(stream), C.byref(out)))
    return out.value


def mebptt_measure_sync(variant: int, iters: int = 3000, stream: Optional[int] = None):
    """(microseconds per synchronisation, status) of the stand-alone synchronisation kernel."""
    out, status = C.c_double(0.0), C.c_int32(0)
    _check(lib().mebptt_measure_sync(variant, iters, _stream(stream), C.byref(out), C.byref(status)))
    return out.value, status.value


def mebptt_bracket_overhead_us(kernel_us: float, reps: int = 200, stream: Optional[int] = None):
    """(time per launch back to back, mean time of the same launch inside its own event pair), in us."""
    a, b = C.c_double(0.0), C.c_double(0.0)
    _check(lib().mebptt_bracket_overhead_us(float(kernel_us), reps, _stream(stream), C.byref(a), C.byref(b)))
    return a.value, b.value


def make_chain_desc(widths, B: int, unit_bytes: int) -> mebptt_chain_desc:
    """Descriptor of a chain of dense tanh layers; keeps the widths array alive on the object."""
    arr = (C.c_int32 * len(widths))(*[int(v) for v in widths])
    d = mebptt_chain_desc(len(widths) - 1, B, arr, unit_bytes)
    d._widths_keepalive = arr
    return d


def mebptt_chain_layers(desc: mebptt_chain_desc):
    """The (cost, state_units, work_units) table of the chain, as mebptt_chain_plan takes it."""
    out = (mebptt_layer * desc.n)()
    _check(lib().mebptt_chain_layers(C.byref(desc), out))
    return [(l.cost, l.state_units, l.work_units) for l in out]


def mebptt_chain_workspace_bytes(desc: mebptt_chain_desc) -> int:
    return lib().mebptt_chain_workspace_bytes(C.byref(desc))


def mebptt_chain_run(desc: mebptt_chain_desc, plan: ChainPlan, W, b, x0, dy, pool, workspace, dW, db, dx0=None,
                     y_out=None, stream: Optional[int] = None) -> mebptt_chain_stats:
    """Enqueues one gradient step of the chain.  W, b, dW, db: lists of n torch tensors (b entries
    may be None); the others torch tensors; `pool` may be None when the plan memorises nothing."""
    n = desc.n
    arr = lambda ts: (_P * n)(*[_ptr(t) for t in ts])
    stats = mebptt_chain_stats()
    rc = lib().mebptt_chain_run(C.byref(desc), plan.handle, arr(W), arr(b), _ptr(x0), _ptr(dy), _ptr(pool),
                                0 if pool is None else _nbytes(pool), _ptr(workspace), _nbytes(workspace), arr(dW),
                                arr(db), _ptr(dx0), _ptr(y_out), C.byref(stats), _stream(stream))
    _check(rc)
    return stats


def mebptt_measure_forward_stream(desc: mebptt_lstm_desc, workspace, reps: int = 50, stream: Optional[int] = None):
    """(us per launch, bytes read per launch) of the kernel that only streams a forward launch's operand panels."""
    a, b = C.c_double(0.0), C.c_double(0.0)
    _check(lib().mebptt_measure_forward_stream(C.byref(desc), _ptr(workspace), _nbytes(workspace), reps, _stream(stream),
                                               C.byref(a), C.byref(b)))
    return a.value, b.value


def mebptt_chunk_steps(desc: mebptt_lstm_desc) -> int:
    n = lib().mebptt_chunk_steps(C.byref(desc))
    if n < 0:
        _check(n)
    return n


def mebptt_stage_steps(desc: mebptt_lstm_desc) -> int:
    n = lib().mebptt_stage_steps(C.byref(desc))
    if n < 0:
        _check(n)
    return n


def mebptt_measure_gemms(desc: mebptt_lstm_desc, workspace, reps: int = 20, stream: Optional[int] = None):
    """(wgrad_us, dgrad_us): the two time-batched GEMMs of one full chunk, alone on the device."""
    a, b = C.c_double(0.0), C.c_double(0.0)
    _check(lib().mebptt_measure_gemms(C.byref(desc), _ptr(workspace), _nbytes(workspace), reps, _stream(stream),
                                      C.byref(a), C.byref(b)))
    return a.value, b.value
