"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Iterable, List, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

SK_F32, SK_BF16, SK_F16 = 0, 1, 2
SK_GEMM, SK_CONV2D_NHWC, SK_CONV2D_NCHW = 0, 1, 2
DTYPE_CODE = {"f32": SK_F32, "bf16": SK_BF16, "f16": SK_F16}
SK_OK, SK_ERR_INVALID_ARG, SK_ERR_UNSUPPORTED, SK_ERR_OVERLAP = 0, -1, -2, -3
SK_ERR_ALLOC, SK_ERR_HIP, SK_ERR_BUSY, SK_ERR_STATE = -4, -5, -6, -7

EXPORTED_SYMBOLS = [
    "sk_plan_params_default", "sk_plan_create", "sk_plan_destroy", "sk_launch", "sk_launch_sequential",
    "sk_launch_static",
    "sk_plan_num_tiles", "sk_plan_num_problems", "sk_plan_get_tiles", "sk_plan_get_order",
    "sk_plan_get_ranges", "sk_plan_grid", "sk_plan_get_xcd_lists", "sk_plan_get_stamps", "sk_release_cached_memory", "sk_strerror", "sk_last_error",
    "sk_queue_params_default", "sk_queue_create", "sk_queue_submit", "sk_queue_poll", "sk_queue_get_stats", "sk_queue_destroy",
]
SK_QUEUE_SEQUENTIAL, SK_QUEUE_COALESCE, SK_QUEUE_OOO = 0, 1, 2
QUEUE_POLICY = {"sequential": SK_QUEUE_SEQUENTIAL, "coalesce": SK_QUEUE_COALESCE, "ooo": SK_QUEUE_OOO}


class SkError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"superkernel status {status}: {detail}")
        self.status = status
        self.detail = detail


class sk_problem(C.Structure):
    _fields_ = [
        ("op", C.c_int32), ("dtype", C.c_int32),
        ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
        ("lda", C.c_int64), ("ldb", C.c_int64), ("ldc", C.c_int64),
        ("Nb", C.c_int32), ("H", C.c_int32), ("Wd", C.c_int32), ("Cin", C.c_int32), ("Cout", C.c_int32),
        ("R", C.c_int32), ("S", C.c_int32), ("pad_h", C.c_int32), ("pad_w", C.c_int32),
        ("stride", C.c_int32),
        ("A", C.c_void_p), ("B", C.c_void_p), ("C", C.c_void_p),
        ("deadline_ms", C.c_double),
    ]


class PlanParams(C.Structure):
    _fields_ = [
        ("edf", C.c_int32), ("stamps", C.c_int32), ("host_only", C.c_int32), ("skinny_max_m", C.c_int32),
        ("tile_bytes_max", C.c_int64), ("tile_bytes_min", C.c_int64),
        ("balance_div", C.c_int32), ("max_groups", C.c_int32), ("grid_limit", C.c_int32),
        ("tail_div", C.c_int32), ("xcd_part", C.c_int32), ("reserved", C.c_int32),
    ]


class QueueParams(C.Structure):
    _fields_ = [("policy", C.c_int32), ("depth", C.c_int32), ("cap_ms", C.c_double), ("bytes_per_ms", C.c_double),
                ("launch_floor_ms", C.c_double)]


class sk_completion(C.Structure):
    _fields_ = [("ticket", C.c_uint64), ("latency_ms", C.c_double), ("budget_ms", C.c_double), ("met", C.c_int32),
                ("launch", C.c_int32)]


class QueueStats(C.Structure):
    _fields_ = [("submitted", C.c_int64), ("completed", C.c_int64), ("launches", C.c_int64), ("met", C.c_int64),
                ("device_busy_ms", C.c_double), ("span_ms", C.c_double)]


def lib_path() -> str:
    """libsuperkernel.so next to this file; SK_LIBRARY names another build of it (the diagnostic one of
    `tile_phases`)."""
    return os.environ.get("SK_LIBRARY") or os.path.join(HERE, "libsuperkernel.so")


_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_1901_10008_amd.build` "
            "(hipcc, gfx950). There is no CPU fallback.")
    L = C.CDLL(path)
    vp = C.c_void_p
    L.sk_plan_params_default.restype = None
    L.sk_plan_params_default.argtypes = [C.POINTER(PlanParams)]
    L.sk_plan_create.restype = C.c_int
    L.sk_plan_create.argtypes = [C.POINTER(sk_problem), C.c_int32, C.POINTER(PlanParams), C.POINTER(vp)]
    L.sk_plan_destroy.restype = C.c_int
    L.sk_plan_destroy.argtypes = [vp]
    for name in ("sk_launch", "sk_launch_sequential", "sk_launch_static"):
        getattr(L, name).restype = C.c_int
        getattr(L, name).argtypes = [vp, vp]
    L.sk_plan_num_tiles.restype = C.c_int64
    L.sk_plan_num_tiles.argtypes = [vp]
    L.sk_plan_num_problems.restype = C.c_int32
    L.sk_plan_num_problems.argtypes = [vp]
    L.sk_plan_grid.restype = C.c_int32
    L.sk_plan_grid.argtypes = [vp]
    L.sk_plan_get_tiles.restype = C.c_int
    L.sk_plan_get_tiles.argtypes = [vp, vp, C.c_int64]
    L.sk_plan_get_order.restype = C.c_int
    L.sk_plan_get_order.argtypes = [vp, C.POINTER(C.c_int32)]
    L.sk_plan_get_xcd_lists.restype = C.c_int
    L.sk_plan_get_xcd_lists.argtypes = [vp, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.c_int64]
    L.sk_plan_get_ranges.restype = C.c_int
    L.sk_plan_get_ranges.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.sk_plan_get_stamps.restype = C.c_int
    L.sk_plan_get_stamps.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_double)]
    L.sk_release_cached_memory.restype = C.c_int
    L.sk_release_cached_memory.argtypes = []
    L.sk_queue_params_default.restype = None
    L.sk_queue_params_default.argtypes = [C.POINTER(QueueParams)]
    L.sk_queue_create.restype = C.c_int
    L.sk_queue_create.argtypes = [C.POINTER(QueueParams), vp, C.POINTER(vp)]
    L.sk_queue_submit.restype = C.c_int
    L.sk_queue_submit.argtypes = [vp, vp, vp, C.c_int32, vp]
    L.sk_queue_poll.restype = C.c_int
    L.sk_queue_poll.argtypes = [vp, C.c_int32, vp, C.c_int32, C.POINTER(C.c_int32)]
    L.sk_queue_get_stats.restype = C.c_int
    L.sk_queue_get_stats.argtypes = [vp, C.POINTER(QueueStats)]
    L.sk_queue_destroy.restype = C.c_int
    L.sk_queue_destroy.argtypes = [vp]
    L.sk_strerror.restype = C.c_char_p
    L.sk_strerror.argtypes = [C.c_int]
    L.sk_last_error.restype = C.c_char_p
    L.sk_last_error.argtypes = []
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        raise SkError(status, (lib().sk_last_error() or b"").decode())


def sk_strerror(status: int) -> str:
    return lib().sk_strerror(status).decode()


def sk_last_error() -> str:
    return (lib().sk_last_error() or b"").decode()


def sk_plan_params_default(**overrides) -> PlanParams:
    p = PlanParams()
    lib().sk_plan_params_default(C.byref(p))
    for k, v in overrides.items():
        if not hasattr(p, k):
            raise AttributeError(k)
        setattr(p, k, v)
    return p


def make_problem(spec, A: int, B: int, Cptr: int, lda: int = 0, ldb: int = 0, ldc: int = 0) -> sk_problem:
    """sk_problem from a description with .op/.dtype/.M/... fields and three device addresses."""
    p = sk_problem()
    p.dtype = DTYPE_CODE[spec.dtype] if isinstance(spec.dtype, str) else int(spec.dtype)
    if spec.op == "gemm":
        p.op = SK_GEMM
        p.M, p.N, p.K = spec.M, spec.N, spec.K
        p.lda, p.ldb, p.ldc = lda, ldb, ldc
    elif spec.op in ("conv", "conv_nchw"):
        p.op = SK_CONV2D_NHWC if spec.op == "conv" else SK_CONV2D_NCHW
        p.Nb, p.H, p.Wd, p.Cin, p.Cout = spec.Nb, spec.H, spec.W, spec.Cin, spec.Cout
        p.R, p.S, p.pad_h, p.pad_w = spec.R, spec.S, spec.pad_h, spec.pad_w
        p.stride = getattr(spec, "stride", 1)
    else:
        raise ValueError(spec.op)
    p.A, p.B, p.C = A, B, Cptr
    d = getattr(spec, "deadline_ms", math.inf)
    p.deadline_ms = float(d) if d is not None else math.inf
    return p


class Plan:
    """Owner of an sk_plan handle (destroyed on close() / garbage collection)."""

    def __init__(self, handle: int, keepalive=None):
        self.handle = handle
        self.keepalive = keepalive

    def close(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().sk_plan_destroy(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def sk_plan_create(problems: Sequence[sk_problem], params: PlanParams | None = None, keepalive=None) -> Plan:
    n = len(problems)
    arr = problems if isinstance(problems, C.Array) else (sk_problem * max(n, 1))(*problems)
    out = C.c_void_p()
    st = lib().sk_plan_create(arr if n else None, n, C.byref(params) if params is not None else None, C.byref(out))
    _check(st)
    return Plan(out.value, keepalive)


def sk_plan_destroy(plan: Plan) -> None:
    plan.close()


def sk_release_cached_memory() -> None:
    _check(lib().sk_release_cached_memory())


def sk_launch(plan: Plan, stream: int = 0) -> None:
    _check(lib().sk_launch(plan.handle, stream))


def sk_launch_sequential(plan: Plan, stream: int = 0) -> None:
    _check(lib().sk_launch_sequential(plan.handle, stream))


def sk_launch_static(plan: Plan, stream: int = 0) -> None:
    _check(lib().sk_launch_static(plan.handle, stream))


SK_STATIC_SCRATCH_BYTES = 32 << 20


def sk_plan_num_tiles(plan: Plan) -> int:
    return int(lib().sk_plan_num_tiles(plan.handle))


def sk_plan_num_problems(plan: Plan) -> int:
    return int(lib().sk_plan_num_problems(plan.handle))


def sk_plan_grid(plan: Plan) -> int:
    return int(lib().sk_plan_grid(plan.handle))


def sk_plan_get_tiles(plan: Plan) -> bytes:
    n = sk_plan_num_tiles(plan)
    buf = C.create_string_buffer(max(32 * n, 1))
    _check(lib().sk_plan_get_tiles(plan.handle, buf, 32 * n))
    return buf.raw[:32 * n]


def sk_plan_get_order(plan: Plan) -> List[int]:
    n = sk_plan_num_problems(plan)
    arr = (C.c_int32 * max(n, 1))()
    _check(lib().sk_plan_get_order(plan.handle, arr))
    return list(arr[:n])


def sk_plan_get_ranges(plan: Plan):
    n = sk_plan_num_problems(plan)
    a = (C.c_int64 * max(n, 1))()
    b = (C.c_int64 * max(n, 1))()
    _check(lib().sk_plan_get_ranges(plan.handle, a, b))
    return list(a[:n]), list(b[:n])


def sk_plan_get_xcd_lists(plan: Plan) -> List[List[int]]:
    """The eight per-die lists of LDS tiles (table indices, in the order the die takes them)."""
    off = (C.c_uint32 * 9)()
    _check(lib().sk_plan_get_xcd_lists(plan.handle, off, None, 0))
    n = int(off[8])
    arr = (C.c_uint32 * max(n, 1))()
    _check(lib().sk_plan_get_xcd_lists(plan.handle, off, arr, n))
    return [list(arr[off[x]:off[x + 1]]) for x in range(8)]


def sk_plan_get_stamps(plan: Plan):
    """(done_ticks[n], start_tick, ticks_per_ms) of the last completed launch."""
    n = sk_plan_num_problems(plan)
    done = (C.c_uint64 * max(n, 1))()
    start = C.c_uint64()
    rate = C.c_double()
    _check(lib().sk_plan_get_stamps(plan.handle, done, C.byref(start), C.byref(rate)))
    return list(done[:n]), int(start.value), float(rate.value)


# ---- operators arriving over time ---------------------------------------------------------------------

def sk_queue_params_default(**overrides) -> QueueParams:
    p = QueueParams()
    lib().sk_queue_params_default(C.byref(p))
    for k, v in overrides.items():
        if not hasattr(p, k):
            raise AttributeError(k)
        setattr(p, k, QUEUE_POLICY[v] if k == "policy" and isinstance(v, str) else v)
    return p


class Queue:
    """Owner of an sk_queue handle."""

    def __init__(self, handle: int, keepalive=None):
        self.handle = handle
        self.keepalive = keepalive
        self._n = C.c_int32()

    def close(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().sk_queue_destroy(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def sk_queue_create(params: QueueParams | None = None, stream: int = 0, keepalive=None) -> Queue:
    out = C.c_void_p()
    _check(lib().sk_queue_create(C.byref(params) if params is not None else None, stream, C.byref(out)))
    return Queue(out.value, keepalive)


def sk_queue_destroy(queue: Queue) -> None:
    queue.close()


def sk_queue_submit(queue: Queue, ops, budgets=None, first: int = 0, n: int | None = None, tickets=None) -> None:
    """Submits ops[first : first + n] (a ctypes array of sk_problem) with budgets[first : first + n] (a ctypes
    array of doubles, or None) and stores their tickets into tickets[first : first + n] (uint64 array or None)."""
    if n is None:
        n = len(ops) - first
    po = C.addressof(ops) + first * C.sizeof(sk_problem)
    pb = C.addressof(budgets) + first * 8 if budgets is not None else None
    pt = C.addressof(tickets) + first * 8 if tickets is not None else None
    _check(lib().sk_queue_submit(queue.handle, po, pb, n, pt))


def sk_queue_poll(queue: Queue, out, wait: bool = False) -> int:
    """Completions into `out` (a ctypes array of sk_completion); returns how many."""
    _check(lib().sk_queue_poll(queue.handle, 1 if wait else 0, C.addressof(out), len(out), C.byref(queue._n)))
    return queue._n.value


def sk_queue_get_stats(queue: Queue) -> QueueStats:
    st = QueueStats()
    _check(lib().sk_queue_get_stats(queue.handle, C.byref(st)))
    return st
