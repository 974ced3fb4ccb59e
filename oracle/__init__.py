"""CPU oracle of the ACCO per-shard optimizer path (TEST INFRASTRUCTURE ONLY).

Thin ctypes access to ``acco_oracle.c`` plus :class:`OracleShard`, which walks the
communication stream of Alg. 1 as one shard owner sees it.  Only ``tests/``, the
smoke check and the bench's ``cpu_baseline`` leg may import this package; it
shares nothing with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

BF16, F32 = 0, 1


class Hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # rebuilt when the source changed; ACCO_SANITIZE=1 selects the ASan + UBSan build
        L = ctypes.CDLL(_build.ensure(_build.selected_so()))
        p, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.oracle_set_threads.argtypes = [ci]
        L.oracle_set_threads.restype = None
        L.oracle_get_threads.restype = ci
        L.oracle_max_threads.restype = ci
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_bf16_to_f32.restype = ctypes.c_float
        L.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.oracle_accumulate.argtypes = [p, p, i64, ci]
        L.oracle_accumulate.restype = None
        L.oracle_accumulate_bf16.argtypes = [p, p, i64, ci]
        L.oracle_accumulate_bf16.restype = None
        L.oracle_cast.argtypes = [p, p, i64]
        L.oracle_cast.restype = None
        L.oracle_reduce.argtypes = [p, ctypes.POINTER(p), ci, ci, i64, ci]
        L.oracle_reduce.restype = None
        for name in ("oracle_estimate_f64", "oracle_estimate_f32"):
            fn = getattr(L, name)
            fn.argtypes = [p, p, p, p, p, p, i64, ctypes.POINTER(Hyper), i64, i64]
            fn.restype = None
        for name in ("oracle_commit_f64", "oracle_commit_f32"):
            fn = getattr(L, name)
            fn.argtypes = [p, p, p, p, p, i64, ctypes.POINTER(Hyper), i64, i64]
            fn.restype = None
        L.oracle_sgd_step.argtypes = [p, p, p, p, i64, ctypes.c_double, ctypes.c_double, i64, ci]
        L.oracle_sgd_step.restype = None
        _lib = L
    return _lib


def set_threads(t: int) -> None:
    lib().oracle_set_threads(int(t))


def usable_cores() -> int:
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        return os.cpu_count() or 1


def make_hyper(lr, beta1, beta2, eps, weight_decay) -> Hyper:
    return Hyper(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay))


def _f32(a: np.ndarray) -> np.ndarray:
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a


def _u16(a: np.ndarray) -> np.ndarray:
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


# --------------------------------------------------------------------------- array calls


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32; exact (numpy view, used by tests)."""
    return (_u16(bits).astype(np.uint32) << 16).view(np.float32)


def accumulate(acc: np.ndarray, grad_bf16: np.ndarray, init: bool) -> None:
    assert acc.shape == grad_bf16.shape
    lib().oracle_accumulate(_f32(acc).ctypes.data, _u16(grad_bf16).ctypes.data, acc.size,
                            int(bool(init)))


def accumulate_bf16(acc_bf16: np.ndarray, grad_bf16: np.ndarray, init: bool) -> None:
    """Running sum held in bf16 (the paper's own buffer precision, Sec. 4)."""
    assert acc_bf16.shape == grad_bf16.shape
    lib().oracle_accumulate_bf16(_u16(acc_bf16).ctypes.data, _u16(grad_bf16).ctypes.data,
                                 acc_bf16.size, int(bool(init)))


def cast(src: np.ndarray) -> np.ndarray:
    out = np.empty(src.shape, dtype=np.uint16)
    lib().oracle_cast(out.ctypes.data, _f32(src).ctypes.data, src.size)
    return out


def reduce(gsum: np.ndarray, shards: Sequence[np.ndarray], accumulate_: bool) -> None:
    W = len(shards)
    assert W >= 1
    dt = BF16 if shards[0].dtype == np.uint16 else F32
    for s in shards:
        assert s.shape == gsum.shape and s.flags.c_contiguous
        assert s.dtype == (np.uint16 if dt == BF16 else np.float32)
    arr = (ctypes.c_void_p * W)(*[s.ctypes.data for s in shards])
    lib().oracle_reduce(_f32(gsum).ctypes.data, arr, W, dt, gsum.size, int(bool(accumulate_)))


def estimate(theta, m, v, gsum, hp: Hyper, step: int, count: int, *, want_f32=True,
             want_bf16=True, precision: str = "f64"):
    n = theta.size
    out_f32 = np.empty(n, np.float32) if want_f32 else None
    out_bf16 = np.empty(n, np.uint16) if want_bf16 else None
    fn = lib().oracle_estimate_f64 if precision == "f64" else lib().oracle_estimate_f32
    fn(_f32(theta).ctypes.data, _f32(m).ctypes.data, _f32(v).ctypes.data, _f32(gsum).ctypes.data,
       _ptr(out_f32), _ptr(out_bf16), n, ctypes.byref(hp), int(step), int(count))
    return out_f32, out_bf16


def commit(theta, m, v, gsum, hp: Hyper, step: int, count: int, *, want_bf16=True,
           precision: str = "f64"):
    """In place on theta, m, v.  Returns the bf16 copy of the new theta (or None)."""
    n = theta.size
    out_bf16 = np.empty(n, np.uint16) if want_bf16 else None
    fn = lib().oracle_commit_f64 if precision == "f64" else lib().oracle_commit_f32
    fn(_f32(theta).ctypes.data, _f32(m).ctypes.data, _f32(v).ctypes.data, _f32(gsum).ctypes.data,
       _ptr(out_bf16), n, ctypes.byref(hp), int(step), int(count))
    return out_bf16


def sgd_step(theta, gsum, lr: float, weight_decay: float, count: int, *, commit: bool,
             want_bf16: bool = True, precision: str = "f64"):
    """Opt = SGD.  commit: in place on theta; else returns the speculative theta as a new array.
    Returns (theta_out, bf16 bits or None)."""
    n = theta.size
    out = theta if commit else np.empty(n, np.float32)
    out_bf16 = np.empty(n, np.uint16) if want_bf16 else None
    lib().oracle_sgd_step(_f32(theta).ctypes.data, _f32(gsum).ctypes.data, out.ctypes.data,
                          _ptr(out_bf16), n, float(lr), float(weight_decay), int(count),
                          int(precision == "f32"))
    return out, out_bf16


def lr_cosine(base_lr: float, min_lr: float, step: int, warmup_steps: int,
              total_steps: int) -> float:
    """Cosine schedule of the paper's hyper-parameter tables with optional linear warm-up:
    the learning rate of update number `step` (0-based)."""
    import math
    if step < warmup_steps:
        return base_lr * (step + 1) / warmup_steps
    span = max(1, total_steps - warmup_steps)
    p = min(1.0, (step - warmup_steps) / span)
    return min_lr + (base_lr - min_lr) * (1.0 + math.cos(math.pi * p)) / 2.0


# --------------------------------------------------------------------------- one shard owner


class OracleShard:
    """State and round sequencing of one shard owner (Alg. 1, communication stream).

    Holds the fp32 shard (theta, m, v), the update index, and per-worker gradient
    accumulators (fp32, or bf16 as in the paper's setup) with their micro-batch counts.  ``precision`` selects
    the binary64 textbook form or the binary32 form of the AdamW update.
    """

    def __init__(self, theta: np.ndarray, workers: int, hp: Hyper, *, m=None, v=None,
                 step: int = 0, precision: str = "f64", comm_dtype: str = "bf16",
                 acc_dtype: str = "f32", lr_schedule=None):
        n = theta.size
        self.n, self.W, self.hp, self.precision = n, workers, hp, precision
        self.lr_schedule = lr_schedule  # step (0-based) -> learning rate of that update
        self.comm_dtype = comm_dtype
        self.acc_dtype = acc_dtype     # "f32" accumulators, or "bf16" as in the paper's setup
        assert acc_dtype in ("f32", "bf16") and (acc_dtype == "f32" or comm_dtype == "bf16")
        self.theta = theta.astype(np.float32, copy=True)
        self.m = np.zeros(n, np.float32) if m is None else m.astype(np.float32, copy=True)
        self.v = np.zeros(n, np.float32) if v is None else v.astype(np.float32, copy=True)
        self.step = int(step)          # number of committed updates so far
        self.acc = [np.zeros(n, np.float32 if acc_dtype == "f32" else np.uint16)
                    for _ in range(workers)]
        self.count = [0] * workers     # micro-batches in each worker's accumulator
        self.gsum = np.zeros(n, np.float32)
        self.total = 0                 # micro-batches summed into gsum
        self.theta_tilde_bf16: Optional[np.ndarray] = None
        self.theta_bf16: Optional[np.ndarray] = None

    def _hp(self) -> Hyper:
        if self.lr_schedule is None:
            return self.hp
        h = self.hp
        return Hyper(float(self.lr_schedule(self.step)), h.beta1, h.beta2, h.eps, h.weight_decay)

    # computation stream: g_i += grad ; N_i += 1
    def add_microbatch(self, worker: int, grad_bf16: np.ndarray) -> None:
        add = accumulate if self.acc_dtype == "f32" else accumulate_bf16
        add(self.acc[worker], grad_bf16, init=(self.count[worker] == 0))
        self.count[worker] += 1

    def _publish(self) -> List[np.ndarray]:
        if self.acc_dtype == "bf16":
            return self.acc            # the accumulator is the communication buffer
        if self.comm_dtype == "bf16":
            return [cast(a) for a in self.acc]
        return self.acc

    # communication stream, stage 1
    def stage1(self) -> None:
        assert all(c >= 1 for c in self.count)
        reduce(self.gsum, self._publish(), accumulate_=False)
        self.total = sum(self.count)                # All_Reduce of the counts
        _, self.theta_tilde_bf16 = estimate(self.theta, self.m, self.v, self.gsum, self._hp(),
                                            self.step + 1, self.total, want_f32=False,
                                            precision=self.precision)
        self.count = [0] * self.W

    # communication stream, stage 2
    def stage2(self) -> None:
        assert all(c >= 1 for c in self.count)
        reduce(self.gsum, self._publish(), accumulate_=True)
        self.total += sum(self.count)
        self.theta_bf16 = commit(self.theta, self.m, self.v, self.gsum, self._hp(), self.step + 1,
                                 self.total, precision=self.precision)
        self.step += 1
        self.count = [0] * self.W
        self.total = 0
