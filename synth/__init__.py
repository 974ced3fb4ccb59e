"""Seeded synthetic inputs for the ACCO shard path, identical on host and device.

This package only manufactures inputs (parameter shards, bf16 micro-batch
gradients, per-worker micro-batch counts).  It contains none of the optimizer
path's arithmetic and is the one module that both the CPU oracle's tests and the
HIP library's tests/bench draw from.  Host fills come from ``libsynth_host.so``
(gcc), device fills from ``libsynth_device.so`` (hipcc, gfx950); both compile the
same ``synth_core.h`` so a slice generated anywhere has the same bits.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

from . import build as _build

# ----------------------------------------------------------------------------- ctypes


class GradSpec(ctypes.Structure):
    _fields_ = [
        ("key", ctypes.c_uint64),
        ("scale", ctypes.c_float),
        ("outlier_scale", ctypes.c_float),
        ("outlier_thr", ctypes.c_uint32),
        ("mask_thr", ctypes.c_uint32),
        ("mask_run", ctypes.c_uint32),
        ("_pad", ctypes.c_uint32),
        ("mask_key", ctypes.c_uint64),
    ]


_host = None
_device = None


def host_lib() -> ctypes.CDLL:
    global _host
    if _host is None:
        # rebuilt when the source changed; ACCO_SANITIZE=1 selects the ASan + UBSan build
        lib = ctypes.CDLL(_build.ensure_host(_build.selected_host_so()))
        lib.synth_host_stream_key.restype = ctypes.c_uint64
        lib.synth_host_stream_key.argtypes = [ctypes.c_uint64] + [ctypes.c_uint32] * 5
        lib.synth_host_hash.restype = ctypes.c_uint64
        lib.synth_host_hash.argtypes = [ctypes.c_uint64, ctypes.c_int64]
        lib.synth_host_ih4_sigma.restype = ctypes.c_double
        for name in ("synth_host_fill_normal_f32", "synth_host_fill_uniform_f32"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64,
                           ctypes.c_float]
        lib.synth_host_fill_grad_bf16.restype = None
        lib.synth_host_fill_grad_bf16.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                  ctypes.POINTER(GradSpec)]
        _host = lib
    return _host


def device_lib() -> ctypes.CDLL:
    """The device fill library; raises if it has not been built (no silent fallback)."""
    global _device
    if _device is None:
        if not os.path.exists(_build.DEVICE_SO):
            raise RuntimeError(f"{_build.DEVICE_SO} is not built; run synth/build.py")
        lib = ctypes.CDLL(_build.DEVICE_SO)
        for name in ("synth_device_fill_normal_f32", "synth_device_fill_uniform_f32"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64,
                           ctypes.c_float, ctypes.c_void_p]
        lib.synth_device_fill_grad_bf16.restype = ctypes.c_int
        lib.synth_device_fill_grad_bf16.argtypes = [ctypes.c_void_p, ctypes.c_int64,
                                                    ctypes.c_int64, ctypes.POINTER(GradSpec),
                                                    ctypes.c_void_p]
        _device = lib
    return _device


# stream kinds
KIND_THETA, KIND_GRAD, KIND_MASK, KIND_COUNT, KIND_WARM = 1, 2, 3, 4, 5
# stages of a round, in the order the shard owner consumes them
STAGE_TILDE, STAGE_FULL = 1, 2


def stream_key(seed: int, kind: int, rnd: int = 0, stage: int = 0, worker: int = 0,
               mb: int = 0) -> int:
    return int(host_lib().synth_host_stream_key(seed, kind, rnd, stage, worker, mb))


def hash64(key: int, j: int) -> int:
    return int(host_lib().synth_host_hash(key, j))


def normal_scale(std: float) -> float:
    """fp32 multiplier that gives the Irwin-Hall(4) lanes the wanted std."""
    return float(np.float32(std / host_lib().synth_host_ih4_sigma()))


def uniform_scale(half_width: float) -> float:
    return float(np.float32(half_width / 16777216.0))


def frac_threshold(p: float) -> int:
    """32-bit threshold t such that P(hash32 < t) = p."""
    return int(min(max(round(p * 4294967296.0), 0), 4294967295))


# ----------------------------------------------------------------------------- host fills


def host_normal_f32(key: int, j0: int, n: int, std: float) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    host_lib().synth_host_fill_normal_f32(out.ctypes.data, j0, n, key, normal_scale(std))
    return out


def host_uniform_f32(key: int, j0: int, n: int, half_width: float) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    host_lib().synth_host_fill_uniform_f32(out.ctypes.data, j0, n, key, uniform_scale(half_width))
    return out


def host_grad_bf16(spec: GradSpec, j0: int, n: int) -> np.ndarray:
    """bf16 bit patterns (uint16) of stream elements j0 .. j0+n-1."""
    out = np.empty(n, dtype=np.uint16)
    host_lib().synth_host_fill_grad_bf16(out.ctypes.data, j0, n, ctypes.byref(spec))
    return out


# ----------------------------------------------------------------------------- device fills


def _stream_ptr():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what}: hipError {rc}")


def device_normal_f32(out, key: int, j0: int, std: float) -> None:
    import torch
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
    _check(device_lib().synth_device_fill_normal_f32(out.data_ptr(), j0, out.numel(), key,
                                                     normal_scale(std), _stream_ptr()),
           "synth_device_fill_normal_f32")


def device_uniform_f32(out, key: int, j0: int, half_width: float) -> None:
    import torch
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
    _check(device_lib().synth_device_fill_uniform_f32(out.data_ptr(), j0, out.numel(), key,
                                                      uniform_scale(half_width), _stream_ptr()),
           "synth_device_fill_uniform_f32")


def device_grad_bf16(out, spec: GradSpec, j0: int) -> None:
    import torch
    assert out.is_cuda and out.dtype == torch.bfloat16 and out.is_contiguous()
    _check(device_lib().synth_device_fill_grad_bf16(out.data_ptr(), j0, out.numel(),
                                                    ctypes.byref(spec), _stream_ptr()),
           "synth_device_fill_grad_bf16")


# ----------------------------------------------------------------------------- workloads


@dataclass(frozen=True)
class Hyper:
    lr: float = 6e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1


@dataclass(frozen=True)
class Workload:
    """One synthetic shard workload: sizes, counts and value distributions.

    A round has two stages.  Stage ``STAGE_TILDE`` carries each worker's first
    ``k_tilde`` micro-batch gradients, stage ``STAGE_FULL`` the remaining ones.
    """
    name: str
    n: int                      # shard length in elements
    workers: int                # W simulated workers
    rounds: int
    seed: int = 0
    theta_dist: str = "normal"  # "normal" (std) or "uniform" (half width)
    theta_param: float = 0.02
    grad_std: float = 1e-4
    zero_frac: float = 0.0      # fraction of elements in all-zero runs
    zero_run: int = 768
    outlier_frac: float = 0.0
    outlier_mult: float = 100.0
    k_fixed: int = 4            # micro-batches per worker per round, if k_range is None
    k_range: Tuple[int, int] | None = None   # inclusive range, drawn per (round, worker)
    warm_steps: int = 0         # optimizer steps taken before round 0 (state from the oracle)
    hyper: Hyper = field(default_factory=Hyper)

    # -- counts
    def microbatches(self, rnd: int, worker: int) -> int:
        if self.k_range is None:
            return self.k_fixed
        lo, hi = self.k_range
        key = stream_key(self.seed, KIND_COUNT, rnd)
        return lo + (hash64(key, worker) >> 33) % (hi - lo + 1)

    def split(self, rnd: int, worker: int) -> Tuple[int, int]:
        """(k_tilde, k_rest): first half rounds down, both >= 1."""
        k = self.microbatches(rnd, worker)
        assert k >= 2
        return k // 2, k - k // 2

    def stage_counts(self, rnd: int, stage: int) -> List[int]:
        idx = 0 if stage == STAGE_TILDE else 1
        return [self.split(rnd, w)[idx] for w in range(self.workers)]

    # -- streams
    def theta_key(self) -> int:
        return stream_key(self.seed, KIND_THETA)

    def grad_spec(self, rnd: int, stage: int, worker: int, mb: int) -> GradSpec:
        sp = GradSpec()
        sp.key = stream_key(self.seed, KIND_GRAD, rnd, stage, worker, mb)
        sp.scale = normal_scale(self.grad_std)
        sp.outlier_scale = normal_scale(self.grad_std * self.outlier_mult)
        sp.outlier_thr = frac_threshold(self.outlier_frac)
        sp.mask_thr = frac_threshold(self.zero_frac)
        sp.mask_run = max(int(self.zero_run), 1)
        sp.mask_key = stream_key(self.seed, KIND_MASK, rnd)
        return sp

    def warm_spec(self, step: int) -> GradSpec:
        """gradient stream of warm-up step `step` (1-based), no mask, same outliers."""
        sp = GradSpec()
        sp.key = stream_key(self.seed, KIND_WARM, step & 0xFFFF, 0, 0, step >> 16)
        sp.scale = normal_scale(self.grad_std)
        sp.outlier_scale = normal_scale(self.grad_std * self.outlier_mult)
        sp.outlier_thr = frac_threshold(self.outlier_frac)
        sp.mask_thr = 0
        sp.mask_run = 1
        sp.mask_key = 0
        return sp

    # -- fills
    def host_theta(self, j0: int, n: int) -> np.ndarray:
        if self.theta_dist == "uniform":
            return host_uniform_f32(self.theta_key(), j0, n, self.theta_param)
        return host_normal_f32(self.theta_key(), j0, n, self.theta_param)

    def device_theta(self, out, j0: int = 0) -> None:
        if self.theta_dist == "uniform":
            device_uniform_f32(out, self.theta_key(), j0, self.theta_param)
        else:
            device_normal_f32(out, self.theta_key(), j0, self.theta_param)

    def sample_slices(self, block: int = 4106, edge: int = 65536) -> List[Tuple[int, int]]:
        """Index ranges [a, b) on which a full-size run is checked element by element:
        the head, the tail (with any ragged remainder) and interior blocks.

        Interior block k starts at k * period, period = 8192 q + 4099 with q chosen so that a
        shard has at least eight interior blocks (q = 2048, about 2^24 elements apart, from
        151M elements on).  The period is odd, so it shares no factor with the power-of-two
        strides of the layouts and launch shapes (vectors of 4 and 8 elements, tiles of 256 to
        8192, state blocks of 8192): the starts walk through all residues, and since
        period mod 8192 = 4099 < block, consecutive blocks cover abutting stretches of the
        8192-element state blocks - every in-block offset is checked within any two consecutive
        samples, and every other sample straddles a state-block boundary."""
        n = self.n
        if n <= (1 << 21):                      # the oracle does such a shard whole in seconds
            return [(0, n)]
        period = max(1, min(2048, n // 9 // 8192)) * 8192 + 4099
        out = [(0, edge)]
        a = period
        while a + block < n - edge:
            out.append((a, a + block))
            a += period
        out.append((n - edge - 37, n))
        return out


def _llm(name, n, workers, rounds, **kw) -> Workload:
    return Workload(name=name, n=n, workers=workers, rounds=rounds, **kw)


WORKLOADS: Dict[str, Workload] = {
    # tiny shard: the oracle finishes it whole in well under a second
    "tiny": _llm("tiny", 1 << 20, 2, 3, theta_dist="uniform", theta_param=0.05,
                 grad_std=1e-3, k_fixed=2),
    # 124,439,808-parameter model (GPT-2-small scale) over 4 owners
    "gpt2s": _llm("gpt2s", 31_109_952, 4, 10, grad_std=1e-3, zero_frac=0.05, k_fixed=8),
    # 1B-parameter model over 8 owners, heavy-tailed gradients, warm optimizer state
    "1b": _llm("1b", 125_000_000, 8, 10, grad_std=1e-4, outlier_frac=1e-3, k_fixed=4,
               warm_steps=100),
    # 7B-parameter model over 8 owners
    "7b": _llm("7b", 875_000_000, 8, 5, grad_std=1e-4, k_fixed=4),
    # heterogeneous worker speeds, ragged shard length
    "7b_hetero": _llm("7b_hetero", 875_000_037, 8, 5, grad_std=1e-4, k_range=(2, 8)),
}
