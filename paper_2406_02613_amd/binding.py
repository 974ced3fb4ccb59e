"""ctypes binding of ``libacco.so`` with the same names as the C ABI (include/acco.h).

Argument marshalling only: tensors are checked (device, dtype, contiguity, length)
and handed to the library as raw device pointers together with torch's current HIP
stream.  Every step of the path runs in the library's kernels; there is no fallback
- if the library is missing the import of this module's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

from . import build as _build

ACCO_OK = 0
ACCO_ERR_NULL, ACCO_ERR_SIZE, ACCO_ERR_ALIGN = -1, -2, -3
ACCO_ERR_ARG, ACCO_ERR_ALIAS, ACCO_ERR_DEVICE = -4, -5, -6
ACCO_BF16, ACCO_F32 = 0, 1
ACCO_MAX_WORKERS = 64
# acco_batch_op
(BATCH_ACCUMULATE_INIT, BATCH_ACCUMULATE, BATCH_ACCUMULATE_PUBLISH, BATCH_FIRST,
 BATCH_FIRST_PUBLISH, BATCH_SECOND, BATCH_SECOND_PUBLISH, BATCH_PUBLISH,
 BATCH_RUNNING_BF16) = range(9)

EXPORTS = ("acco_accumulate", "acco_accumulate_publish", "acco_accumulate_first",
           "acco_accumulate_second", "acco_accumulate_bf16", "acco_accumulate_batch",
           "acco_cast_params", "acco_reduce_shards",
           "acco_estimate_step", "acco_commit_step", "acco_reduce_estimate_step",
           "acco_reduce_commit_step", "acco_fold_adamw", "acco_stage_scalars",
           "acco_estimate_step_dev", "acco_commit_step_dev", "acco_reduce_estimate_step_dev",
           "acco_reduce_commit_step_dev", "acco_commit_step_resident",
           "acco_sgd_estimate_step", "acco_sgd_commit_step",
           "acco_lr_cosine", "acco_hbm_classify", "acco_probe_copy", "acco_probe_triad", "acco_status_string", "acco_version", "acco_set_launch_shape",
           "acco_set_resident_waves", "acco_reset_launch_settings")


class AdamW(ctypes.Structure):
    """acco_adamw_t"""
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double)]


class Layout(ctypes.Structure):
    """acco_layout_t"""
    _fields_ = [("block_elems", ctypes.c_int64), ("block_stride", ctypes.c_int64)]


class Sgd(ctypes.Structure):
    """acco_sgd_t"""
    _fields_ = [("lr", ctypes.c_double), ("weight_decay", ctypes.c_double)]


class StepScalars(ctypes.Structure):
    """acco_step_scalars_t: one step's folded scalars (opaque, 64 bytes)"""
    _fields_ = [("f", ctypes.c_float * 16)]


STAGE_BLOCKS_MAX = 4


class AccoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        so = _build.selected_so()
        if not os.path.exists(so):
            raise RuntimeError(
                f"{so} not found: build it with paper_2406_02613_amd/build.py "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(so)
        p, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        pi64 = ctypes.POINTER(ctypes.c_int64)
        play = ctypes.POINTER(Layout)
        L.acco_accumulate.argtypes = [p, p, i64, ci, pi64, p]
        L.acco_cast_params.argtypes = [p, p, i64, p]
        L.acco_reduce_shards.argtypes = [p, ctypes.POINTER(p), ci, ci, i64, ci, pi64, pi64, play, play,
                                         p]
        L.acco_estimate_step.argtypes = [p, p, p, p, p, p, i64, ctypes.POINTER(AdamW), i64, i64,
                                         play, p]
        L.acco_commit_step.argtypes = [p, p, p, p, p, i64, ctypes.POINTER(AdamW), pi64, i64, play,
                                       p]
        L.acco_accumulate_publish.argtypes = [p, p, p, i64, ci, ci, pi64, p]
        L.acco_accumulate_first.argtypes = [p, p, i64, ci, pi64, p]
        L.acco_accumulate_bf16.argtypes = [p, p, i64, ci, pi64, p]
        L.acco_accumulate_second.argtypes = [p, p, p, p, i64, pi64, p]
        pp = ctypes.POINTER(p)
        L.acco_accumulate_batch.argtypes = [ci, ci, pp, pp, pp, pp, i64, pi64, play, p]
        L.acco_reduce_estimate_step.argtypes = [p, p, p, p, ctypes.POINTER(p), ci, ci, pi64, pi64,
                                                p, p, i64, ctypes.POINTER(AdamW), i64, play, play,
                                                p]
        L.acco_reduce_commit_step.argtypes = [p, p, p, p, ctypes.POINTER(p), ci, ci, pi64, pi64, p,
                                              i64, ctypes.POINTER(AdamW), pi64, play, play, p]
        psc = ctypes.POINTER(StepScalars)
        L.acco_fold_adamw.argtypes = [ctypes.POINTER(AdamW), i64, i64, psc]
        L.acco_stage_scalars.argtypes = [p, psc, ci, p]
        L.acco_estimate_step_dev.argtypes = [p, p, p, p, p, i64, p, play, p]
        L.acco_commit_step_dev.argtypes = [p, p, p, p, p, i64, p, play, p]
        L.acco_reduce_estimate_step_dev.argtypes = [p, p, p, p, ctypes.POINTER(p), ci, ci, p, i64,
                                                    p, play, play, p]
        L.acco_reduce_commit_step_dev.argtypes = [p, p, p, p, ctypes.POINTER(p), ci, ci, p, i64, p,
                                                  play, play, p]
        L.acco_commit_step_resident.argtypes = [p, p, p, p, p, i64, psc, ci, play, p]
        L.acco_sgd_estimate_step.argtypes = [p, p, p, p, i64, ctypes.POINTER(Sgd), i64, p]
        L.acco_sgd_commit_step.argtypes = [p, p, p, i64, ctypes.POINTER(Sgd), pi64, i64, p]
        L.acco_set_launch_shape.argtypes = [ctypes.c_char_p, ci, ci, ci]
        L.acco_set_resident_waves.argtypes = [ctypes.c_char_p, ci]
        for name in EXPORTS:
            getattr(L, name).restype = ci
        L.acco_reset_launch_settings.argtypes = []
        L.acco_reset_launch_settings.restype = None
        L.acco_hbm_classify.argtypes = [p, i64, i64, i64, p, ctypes.POINTER(ctypes.c_int32), i64,
                                        ctypes.POINTER(ctypes.c_int32), p]
        L.acco_probe_copy.argtypes = [p, p, i64, p]
        L.acco_probe_triad.argtypes = [p, p, p, p, i64, p]
        L.acco_lr_cosine.restype = ctypes.c_double
        L.acco_lr_cosine.argtypes = [ctypes.c_double, ctypes.c_double, i64, i64, i64]
        L.acco_status_string.restype = ctypes.c_char_p
        L.acco_status_string.argtypes = [ci]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().acco_status_string(int(status)).decode()


def version() -> int:
    return int(lib().acco_version())


def set_launch_shape(entry: str, threads: int, vectors_in_flight: int,
                     workgroups_per_cu: int) -> None:
    rc = lib().acco_set_launch_shape(entry.encode(), threads, vectors_in_flight, workgroups_per_cu)
    if rc != ACCO_OK:
        raise AccoError(rc, "acco_set_launch_shape")


def reset_launch_settings() -> None:
    lib().acco_reset_launch_settings()


def set_resident_waves(entry: str, waves_per_cu: int) -> None:
    rc = lib().acco_set_resident_waves(entry.encode(), waves_per_cu)
    if rc != ACCO_OK:
        raise AccoError(rc, "acco_set_resident_waves")


# ----------------------------------------------------------------------------- marshalling


def _stream() -> ctypes.c_void_p:
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, n: int, name: str) -> int:
    """Device pointer of a checked tensor."""
    import torch
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: expected a torch.Tensor")
    if not t.is_cuda:
        raise ValueError(f"{name}: must live on the GPU")
    if t.device.index != torch.cuda.current_device():
        raise ValueError(f"{name}: is on {t.device}, current device is "
                         f"{torch.cuda.current_device()}")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if t.numel() != n:
        raise ValueError(f"{name}: has {t.numel()} elements, expected {n}")
    return t.data_ptr()


def _state(tensors, names, n=None, dtype=None):
    """Pointers, logical length and layout of arrays that share a layout (theta, m, v, gsum; or
    the workers' communication buffers).

    Each tensor is either 1-D contiguous (planar) or a 2-D view of shape (blocks, block_elems)
    with strides (block_stride, 1) - a component of a block-interleaved buffer.  All tensors
    passed together must have the same form.  dtype: torch.float32 unless given."""
    import torch
    dtype = torch.float32 if dtype is None else dtype
    t0 = tensors[0]
    if t0.dim() == 1:
        n = t0.numel() if n is None else int(n)
        return [_dev(t, dtype, n, nm) for t, nm in zip(tensors, names)], n, None
    if t0.dim() != 2:
        raise ValueError(f"{names[0]}: expected a 1-D tensor or a (blocks, block_elems) view")
    nblk, blk = t0.shape
    stride = t0.stride(0)
    n = nblk * blk if n is None else int(n)
    lo = (nblk - 1) * blk if nblk else -1
    if not lo < n <= nblk * blk:
        raise ValueError(f"n={n} does not fit {nblk} blocks of {blk}")
    ptrs = []
    for t, nm in zip(tensors, names):
        if not t.is_cuda or t.device.index != torch.cuda.current_device():
            raise ValueError(f"{nm}: must live on the current GPU")
        if t.dtype != dtype:
            raise TypeError(f"{nm}: expected {dtype}, got {t.dtype}")
        if t.dim() != 2 or tuple(t.shape) != (nblk, blk) or t.stride(1) != 1 or \
                (nblk > 1 and t.stride(0) != stride):
            raise ValueError(f"{nm}: all state views must share shape (blocks, block_elems) and "
                             "strides (block_stride, 1)")
        ptrs.append(t.data_ptr())
    return ptrs, n, Layout(blk, stride)


def _lay(layout):
    return None if layout is None else ctypes.byref(layout)


def _opt(t, dtype, n, name):
    return None if t is None else _dev(t, dtype, n, name)


def _check(rc: int, where: str) -> None:
    if rc != ACCO_OK:
        raise AccoError(rc, where)


class Counter:
    """A host int64 the library reads and updates (micro-batch counts, totals, step)."""

    def __init__(self, value: int = 0):
        self._c = ctypes.c_int64(int(value))

    @property
    def value(self) -> int:
        return int(self._c.value)

    @value.setter
    def value(self, x: int) -> None:
        self._c.value = int(x)

    def ref(self):
        return ctypes.byref(self._c)

    def __repr__(self) -> str:
        return f"Counter({self.value})"


def make_hyper(lr, beta1, beta2, eps, weight_decay) -> AdamW:
    return AdamW(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay))


# ----------------------------------------------------------------------------- entry points


def acco_accumulate(acc, grad_bf16, init: bool, count: Optional[Counter] = None) -> None:
    import torch
    n = acc.numel()
    rc = lib().acco_accumulate(_dev(acc, torch.float32, n, "acc"),
                               _dev(grad_bf16, torch.bfloat16, n, "grad_bf16"), n,
                               int(bool(init)), None if count is None else count.ref(), _stream())
    _check(rc, "acco_accumulate")


def acco_accumulate_bf16(acc_bf16, grad_bf16, init: bool, count: Optional[Counter] = None) -> None:
    import torch
    n = grad_bf16.numel()
    rc = lib().acco_accumulate_bf16(_dev(acc_bf16, torch.bfloat16, n, "acc_bf16"),
                                    _dev(grad_bf16, torch.bfloat16, n, "grad_bf16"), n,
                                    int(bool(init)), None if count is None else count.ref(),
                                    _stream())
    _check(rc, "acco_accumulate_bf16")


def acco_accumulate_publish(acc, grad_bf16, comm_bf16, init: bool, keep_acc: bool = False,
                            count: Optional[Counter] = None) -> None:
    import torch
    n = grad_bf16.numel()
    acc_ptr = None if (acc is None) else _dev(acc, torch.float32, n, "acc")
    rc = lib().acco_accumulate_publish(acc_ptr, _dev(grad_bf16, torch.bfloat16, n, "grad_bf16"),
                                       _dev(comm_bf16, torch.bfloat16, n, "comm_bf16"), n,
                                       int(bool(init)), int(bool(keep_acc)),
                                       None if count is None else count.ref(), _stream())
    _check(rc, "acco_accumulate_publish")


def acco_accumulate_first(stash_bf16, grad_bf16, publish: bool = False,
                          count: Optional[Counter] = None) -> None:
    import torch
    n = grad_bf16.numel()
    rc = lib().acco_accumulate_first(_dev(stash_bf16, torch.bfloat16, n, "stash_bf16"),
                                     _dev(grad_bf16, torch.bfloat16, n, "grad_bf16"), n,
                                     int(bool(publish)), None if count is None else count.ref(),
                                     _stream())
    _check(rc, "acco_accumulate_first")


def acco_accumulate_second(stash_bf16, grad_bf16, *, acc=None, comm_bf16=None,
                           count: Optional[Counter] = None) -> None:
    import torch
    n = grad_bf16.numel()
    rc = lib().acco_accumulate_second(_opt(acc, torch.float32, n, "acc"),
                                      _opt(comm_bf16, torch.bfloat16, n, "comm_bf16"),
                                      _dev(stash_bf16, torch.bfloat16, n, "stash_bf16"),
                                      _dev(grad_bf16, torch.bfloat16, n, "grad_bf16"), n,
                                      None if count is None else count.ref(), _stream())
    _check(rc, "acco_accumulate_second")


def acco_accumulate_batch(op: int, n: int, *, acc: Optional[Sequence] = None,
                          out_bf16: Optional[Sequence] = None,
                          stash_bf16: Optional[Sequence] = None,
                          grad_bf16: Optional[Sequence] = None,
                          counts: Optional[Sequence[Counter]] = None) -> None:
    """One accumulation step of several workers in one launch; each array argument is a
    sequence with one tensor per worker.  out_bf16 may be planar tensors or the views of an
    interleaved buffer (state.InterleavedShards); the layout is derived from their strides.
    The workers' counters are updated as by the single calls."""
    import torch
    cols = (("acc", acc, torch.float32), ("out_bf16", out_bf16, torch.bfloat16),
            ("stash_bf16", stash_bf16, torch.bfloat16), ("grad_bf16", grad_bf16, torch.bfloat16))
    W = max(len(c) for _, c, _ in cols if c is not None)
    arrays, layout = [], None
    for name, col, dt in cols:
        if col is None:
            arrays.append(None)
            continue
        if len(col) != W:
            raise ValueError(f"{name}: one tensor per worker")
        if name == "out_bf16":
            ptrs, _, layout = _state(list(col), [f"{name}[{i}]" for i in range(W)], n, dt)
        else:
            ptrs = [_dev(t, dt, n, f"{name}[{i}]") for i, t in enumerate(col)]
        arrays.append((ctypes.c_void_p * W)(*ptrs))
    cnts = None
    if counts is not None:
        if len(counts) != W:
            raise ValueError("counts: one per worker")
        cnts = (ctypes.c_int64 * W)(*[c.value for c in counts])
    rc = lib().acco_accumulate_batch(int(op), W, *arrays, int(n), cnts, _lay(layout), _stream())
    _check(rc, "acco_accumulate_batch")
    if counts is not None:
        for c, x in zip(counts, cnts):
            c.value = x


def acco_cast_params(out_bf16, src) -> None:
    import torch
    n = src.numel()
    rc = lib().acco_cast_params(_dev(out_bf16, torch.bfloat16, n, "out_bf16"),
                                _dev(src, torch.float32, n, "src"), n, _stream())
    _check(rc, "acco_cast_params")


def _shard_ptrs(shards: Sequence, n: int, where: str):
    """Device pointers, dtype code and layout of the worker shards (planar tensors or the views
    of an interleaved bf16 buffer)."""
    import torch
    W = len(shards)
    if W < 1:
        raise AccoError(ACCO_ERR_SIZE, where)
    dt = shards[0].dtype
    if dt not in (torch.bfloat16, torch.float32):
        raise TypeError("shards: expected bfloat16 or float32 tensors")
    ptrs, _, layout = _state(list(shards), [f"shards[{i}]" for i in range(W)], n, dt)
    return ((ctypes.c_void_p * W)(*ptrs), W, ACCO_BF16 if dt == torch.bfloat16 else ACCO_F32,
            layout)


def acco_reduce_shards(gsum, shards: Sequence, accumulate: bool,
                       counts: Optional[Sequence[int]] = None,
                       total: Optional[Counter] = None, n: Optional[int] = None) -> None:
    (gsum_ptr,), n, layout = _state([gsum], ["gsum"], n)
    ptrs, W, dt, shard_layout = _shard_ptrs(shards, n, "acco_reduce_shards")
    cnts = None
    if counts is not None:
        if len(counts) != W:
            raise ValueError("counts: one per shard")
        cnts = (ctypes.c_int64 * W)(*[int(c) for c in counts])
    rc = lib().acco_reduce_shards(gsum_ptr, ptrs, W, dt, n, int(bool(accumulate)), cnts,
                                  None if total is None else total.ref(), _lay(layout),
                                  _lay(shard_layout), _stream())
    _check(rc, "acco_reduce_shards")


def _shard_args(shards: Sequence, n: int, counts: Sequence[int], where: str):
    ptrs, W, dt, shard_layout = _shard_ptrs(shards, n, where)
    if len(counts) != W:
        raise ValueError("counts: one per shard")
    cnts = (ctypes.c_int64 * W)(*[int(c) for c in counts])
    return ptrs, cnts, W, dt, shard_layout


def acco_reduce_estimate_step(theta, m, v, gsum, shards: Sequence, counts: Sequence[int],
                              total: Counter, hp: AdamW, step: int, *, theta_tilde_f32=None,
                              theta_tilde_bf16=None, n: Optional[int] = None) -> None:
    import torch
    f32 = torch.float32
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    ptrs, cnts, W, dt, sl = _shard_args(shards, n, counts, "acco_reduce_estimate_step")
    rc = lib().acco_reduce_estimate_step(
        st[0], st[1], st[2], st[3], ptrs, W, dt, cnts, total.ref(),
        _opt(theta_tilde_f32, f32, n, "theta_tilde_f32"),
        _opt(theta_tilde_bf16, torch.bfloat16, n, "theta_tilde_bf16"), n, ctypes.byref(hp),
        int(step), _lay(layout), _lay(sl), _stream())
    _check(rc, "acco_reduce_estimate_step")


def acco_reduce_commit_step(theta, m, v, gsum, shards: Sequence, counts: Sequence[int],
                            total: Counter, hp: AdamW, step: Counter, *, theta_bf16=None,
                            n: Optional[int] = None) -> None:
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    ptrs, cnts, W, dt, sl = _shard_args(shards, n, counts, "acco_reduce_commit_step")
    rc = lib().acco_reduce_commit_step(
        st[0], st[1], st[2], st[3], ptrs, W, dt, cnts, total.ref(),
        _opt(theta_bf16, torch.bfloat16, n, "theta_bf16"), n, ctypes.byref(hp), step.ref(),
        _lay(layout), _lay(sl), _stream())
    _check(rc, "acco_reduce_commit_step")


def acco_estimate_step(theta, m, v, gsum, hp: AdamW, step: int, total_count: int, *,
                       theta_tilde_f32=None, theta_tilde_bf16=None,
                       n: Optional[int] = None) -> None:
    import torch
    f32 = torch.float32
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    rc = lib().acco_estimate_step(st[0], st[1], st[2], st[3],
                                  _opt(theta_tilde_f32, f32, n, "theta_tilde_f32"),
                                  _opt(theta_tilde_bf16, torch.bfloat16, n, "theta_tilde_bf16"),
                                  n, ctypes.byref(hp), int(step), int(total_count), _lay(layout),
                                  _stream())
    _check(rc, "acco_estimate_step")


def acco_commit_step(theta, m, v, gsum, hp: AdamW, step: Counter, total_count: int, *,
                     theta_bf16=None, n: Optional[int] = None) -> None:
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    rc = lib().acco_commit_step(st[0], st[1], st[2], st[3],
                                _opt(theta_bf16, torch.bfloat16, n, "theta_bf16"), n,
                                ctypes.byref(hp), step.ref(), int(total_count), _lay(layout),
                                _stream())
    _check(rc, "acco_commit_step")


# ------------------------------------------------- step scalars in device memory (*_dev forms)


def acco_fold_adamw(hp: AdamW, step: int, total_count: int) -> StepScalars:
    """Folded scalars of update number step + 1 on a sum of total_count micro-batch gradients."""
    out = StepScalars()
    _check(lib().acco_fold_adamw(ctypes.byref(hp), int(step), int(total_count), ctypes.byref(out)),
           "acco_fold_adamw")
    return out


def _scalars_ptr(scalars_dev, block: int) -> int:
    """Address of block `block` of a device tensor of scalar blocks (float32, 16 per block)."""
    import torch
    nblk = scalars_dev.numel() // 16
    if scalars_dev.numel() % 16 or not 0 <= int(block) < nblk:
        raise ValueError("scalars_dev: expected 16 float32 per block and a block inside it")
    return _dev(scalars_dev, torch.float32, scalars_dev.numel(), "scalars_dev") + 64 * int(block)


def acco_stage_scalars(scalars_dev, blocks: Sequence[StepScalars], first_block: int = 0) -> None:
    """scalars_dev[first_block ...] = blocks, by one small kernel on the current stream."""
    k = len(blocks)
    _scalars_ptr(scalars_dev, first_block + k - 1 if k else first_block)
    src = (StepScalars * max(k, 1))(*blocks)
    _check(lib().acco_stage_scalars(_scalars_ptr(scalars_dev, first_block), src, k, _stream()),
           "acco_stage_scalars")


class ScalarStager:
    """acco_fold_adamw + acco_stage_scalars for the first `blocks` blocks of one device tensor,
    with the tensor checked and the argument arrays built once: for loops that restage the
    scalars before every replay of a recorded round."""

    def __init__(self, scalars_dev, blocks: int):
        if not 1 <= int(blocks) <= STAGE_BLOCKS_MAX:
            raise ValueError(f"1 to {STAGE_BLOCKS_MAX} blocks per call")
        _scalars_ptr(scalars_dev, int(blocks) - 1)
        self._keep = scalars_dev
        self._ptr = ctypes.c_void_p(_scalars_ptr(scalars_dev, 0))
        self._k = int(blocks)
        self._src = (StepScalars * self._k)()
        self._lib = lib()

    def __call__(self, hp: AdamW, step: int, totals: Sequence[int]) -> None:
        """Block k <- the scalars of update number step + 1 on totals[k] micro-batches."""
        if len(totals) != self._k:
            raise ValueError("one total per block")
        L, hp_ref = self._lib, ctypes.byref(hp)
        for k, t in enumerate(totals):
            _check(L.acco_fold_adamw(hp_ref, int(step), int(t), ctypes.byref(self._src[k])),
                   "acco_fold_adamw")
        _check(L.acco_stage_scalars(self._ptr, self._src, self._k, _stream()),
               "acco_stage_scalars")


def acco_estimate_step_dev(theta, m, v, gsum, scalars_dev, block: int, *, theta_tilde_bf16,
                           n: Optional[int] = None) -> None:
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    rc = lib().acco_estimate_step_dev(st[0], st[1], st[2], st[3],
                                      _dev(theta_tilde_bf16, torch.bfloat16, n, "theta_tilde_bf16"),
                                      n, _scalars_ptr(scalars_dev, block), _lay(layout), _stream())
    _check(rc, "acco_estimate_step_dev")


def acco_commit_step_dev(theta, m, v, gsum, scalars_dev, block: int, *, theta_bf16=None,
                         n: Optional[int] = None) -> None:
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    rc = lib().acco_commit_step_dev(st[0], st[1], st[2], st[3],
                                    _opt(theta_bf16, torch.bfloat16, n, "theta_bf16"), n,
                                    _scalars_ptr(scalars_dev, block), _lay(layout), _stream())
    _check(rc, "acco_commit_step_dev")


def acco_reduce_estimate_step_dev(theta, m, v, gsum, shards: Sequence, scalars_dev, block: int, *,
                                  theta_tilde_bf16, n: Optional[int] = None) -> None:
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    ptrs, W, dt, sl = _shard_ptrs(shards, n, "acco_reduce_estimate_step_dev")
    rc = lib().acco_reduce_estimate_step_dev(
        st[0], st[1], st[2], st[3], ptrs, W, dt,
        _dev(theta_tilde_bf16, torch.bfloat16, n, "theta_tilde_bf16"), n,
        _scalars_ptr(scalars_dev, block), _lay(layout), _lay(sl), _stream())
    _check(rc, "acco_reduce_estimate_step_dev")


def acco_reduce_commit_step_dev(theta, m, v, gsum, shards: Sequence, scalars_dev, block: int, *,
                                theta_bf16=None, n: Optional[int] = None) -> None:
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    ptrs, W, dt, sl = _shard_ptrs(shards, n, "acco_reduce_commit_step_dev")
    rc = lib().acco_reduce_commit_step_dev(
        st[0], st[1], st[2], st[3], ptrs, W, dt,
        _opt(theta_bf16, torch.bfloat16, n, "theta_bf16"), n, _scalars_ptr(scalars_dev, block),
        _lay(layout), _lay(sl), _stream())
    _check(rc, "acco_reduce_commit_step_dev")


RESIDENT_SLOTS = 64


def acco_commit_step_resident(theta, m, v, gsum, scalars: StepScalars, slot: int, *,
                              theta_bf16=None, n: Optional[int] = None) -> None:
    """acco_commit_step_dev with the scalar block held by the library (nothing to allocate)."""
    import torch
    st, n, layout = _state([theta, m, v, gsum], ["theta", "m", "v", "gsum"], n)
    rc = lib().acco_commit_step_resident(st[0], st[1], st[2], st[3],
                                         _opt(theta_bf16, torch.bfloat16, n, "theta_bf16"), n,
                                         ctypes.byref(scalars), int(slot), _lay(layout), _stream())
    _check(rc, "acco_commit_step_resident")


def make_sgd(lr, weight_decay=0.0) -> Sgd:
    return Sgd(float(lr), float(weight_decay))


def acco_sgd_estimate_step(theta, gsum, hp: Sgd, total_count: int, *, theta_tilde_f32=None,
                           theta_tilde_bf16=None) -> None:
    import torch
    n = theta.numel()
    f32 = torch.float32
    rc = lib().acco_sgd_estimate_step(_dev(theta, f32, n, "theta"), _dev(gsum, f32, n, "gsum"),
                                      _opt(theta_tilde_f32, f32, n, "theta_tilde_f32"),
                                      _opt(theta_tilde_bf16, torch.bfloat16, n, "theta_tilde_bf16"),
                                      n, ctypes.byref(hp), int(total_count), _stream())
    _check(rc, "acco_sgd_estimate_step")


def acco_sgd_commit_step(theta, gsum, hp: Sgd, step: Counter, total_count: int, *,
                         theta_bf16=None) -> None:
    import torch
    n = theta.numel()
    f32 = torch.float32
    rc = lib().acco_sgd_commit_step(_dev(theta, f32, n, "theta"), _dev(gsum, f32, n, "gsum"),
                                    _opt(theta_bf16, torch.bfloat16, n, "theta_bf16"), n,
                                    ctypes.byref(hp), step.ref(), int(total_count), _stream())
    _check(rc, "acco_sgd_commit_step")


def acco_lr_cosine(base_lr: float, min_lr: float, step: int, warmup_steps: int,
                   total_steps: int) -> float:
    return float(lib().acco_lr_cosine(float(base_lr), float(min_lr), int(step), int(warmup_steps),
                                      int(total_steps)))


def acco_hbm_classify(region, step_bytes: int, probe_bytes: int, scratch):
    """Memory class of every position of `region` (a contiguous uint8 device tensor):
    (classes, n_classes), classes[k] for the probe_bytes at offset k * step_bytes."""
    import torch
    nbytes = region.numel()
    base = _dev(region, torch.uint8, nbytes, "region")
    count = (nbytes - int(probe_bytes)) // int(step_bytes) + 1 if nbytes >= probe_bytes else 0
    out = (ctypes.c_int32 * max(count, 1))()
    ncls = ctypes.c_int32(0)
    rc = lib().acco_hbm_classify(base, nbytes, int(step_bytes), int(probe_bytes),
                                 _dev(scratch, torch.uint8, int(probe_bytes), "scratch"), out,
                                 count, ctypes.byref(ncls), _stream())
    _check(rc, "acco_hbm_classify")
    return list(out[:count]), int(ncls.value)


def acco_probe_copy(dst, src) -> None:
    import torch
    n = src.numel()
    _check(lib().acco_probe_copy(_dev(dst, torch.float32, n, "dst"),
                                 _dev(src, torch.float32, n, "src"), n, _stream()),
           "acco_probe_copy")


def acco_probe_triad(a, b, c, d) -> None:
    import torch
    n = a.numel()
    f32 = torch.float32
    _check(lib().acco_probe_triad(_dev(a, f32, n, "a"), _dev(b, f32, n, "b"), _dev(c, f32, n, "c"),
                                  _dev(d, f32, n, "d"), n, _stream()), "acco_probe_triad")
