"""Shared helpers of the GPU parity tests (not a test module)."""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

import oracle
import synth

TOL_REL, TOL_ABS = 2e-6, 1e-9          # fp32 theta / m / v: relative, or absolute
BF16_MAX_ULP = 1                       # bf16 outputs


def oracle_hyper(w: synth.Workload):
    h = w.hyper
    return oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay)


def bits_of(t) -> np.ndarray:
    """bf16 torch tensor (any device) -> uint16 bit patterns on the host."""
    import torch
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_tensor(bits: np.ndarray, device="cuda"):
    import torch
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(device)


def f32_close(got: np.ndarray, want: np.ndarray, rel=TOL_REL, abs_=TOL_ABS) -> Tuple[bool, str]:
    g = got.astype(np.float64)
    w = want.astype(np.float64)
    nan_ok = np.isnan(g) == np.isnan(w)
    err = np.abs(g - w)
    err = np.where(np.isnan(w), 0.0, err)
    ok = ((err <= abs_) | (err <= rel * np.abs(w)) | (g == w)) & nan_ok
    if ok.all():
        return True, ""
    i = int(np.argmax(~ok))
    return False, (f"{int((~ok).sum())} of {ok.size} outside tolerance; first at {i}: "
                   f"got {got[i]!r} want {want[i]!r}")


def assert_f32_close(got, want, what="", **kw):
    ok, msg = f32_close(np.asarray(got), np.asarray(want), **kw)
    assert ok, f"{what}: {msg}"


def bit_mismatches(got: np.ndarray, want: np.ndarray) -> int:
    return int(np.count_nonzero(got.view(np.uint32) != want.view(np.uint32)))


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def assert_bf16_close(got_bits, want_bits, what=""):
    """bf16 outputs: at most one bf16 ulp apart.  Where the fp32 value underneath is so small
    that its own tolerance is the absolute one (1e-9, e.g. theta cancelling against the Adam
    step), one ulp of such a value is far below that tolerance, so the same absolute tolerance
    (plus the two bf16 roundings) applies to the bf16 values."""
    both_nan = ((got_bits & 0x7FFF) > 0x7F80) & ((want_bits & 0x7FFF) > 0x7F80)
    d = np.where(both_nan, 0, bf16_ulp_distance(got_bits, want_bits))
    gv = oracle.bf16_to_f32(np.ascontiguousarray(got_bits)).astype(np.float64)
    wv = oracle.bf16_to_f32(np.ascontiguousarray(want_bits)).astype(np.float64)
    with np.errstate(invalid="ignore"):
        tiny = np.abs(gv - wv) <= TOL_ABS + 2.0 ** -8 * np.maximum(np.abs(gv), np.abs(wv))
        tiny &= np.maximum(np.abs(gv), np.abs(wv)) <= 1e-6
    bad = (d > BF16_MAX_ULP) & ~tiny
    assert not bad.any(), (
        f"{what}: bf16 differs by {int(d[bad].max())} ulp at {int(np.argmax(bad))}: "
        f"{gv[np.argmax(bad)]!r} vs {wv[np.argmax(bad)]!r}")


# ------------------------------------------------------------------ oracle runs on slices


def oracle_warm_state(w: synth.Workload, j0: int, n: int, chunk: int = 1 << 20):
    """theta, m, v of elements [j0, j0+n) after w.warm_steps plain committed updates, each on
    one synthetic gradient (count 1), computed by the oracle (binary64 form)."""
    theta = w.host_theta(j0, n)
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    hp = oracle_hyper(w)
    specs = [w.warm_spec(s) for s in range(1, w.warm_steps + 1)]
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        th, mm, vv = theta[a:b], m[a:b], v[a:b]      # contiguous views, updated in place
        g = np.empty(b - a, np.float32)
        for s, sp in enumerate(specs, start=1):
            oracle.accumulate(g, synth.host_grad_bf16(sp, j0 + a, b - a), init=True)
            oracle.commit(th, mm, vv, g, hp, step=s, count=1, want_bf16=False)
    return theta, m, v


class OracleSlices:
    """The oracle run on a list of index ranges of a workload, one OracleShard per range."""

    def __init__(self, w: synth.Workload, slices: Sequence[Tuple[int, int]], precision: str,
                 comm_dtype: str = "bf16", warm=None, acc_dtype: str = "f32"):
        self.w, self.slices = w, list(slices)
        self.shards: List[oracle.OracleShard] = []
        for k, (a, b) in enumerate(self.slices):
            if warm is not None:
                th, m, v = (x[a:b] for x in warm)
                sh = oracle.OracleShard(th, w.workers, oracle_hyper(w), m=m, v=v,
                                        step=w.warm_steps, precision=precision,
                                        comm_dtype=comm_dtype, acc_dtype=acc_dtype)
            else:
                sh = oracle.OracleShard(w.host_theta(a, b - a), w.workers, oracle_hyper(w),
                                        precision=precision, comm_dtype=comm_dtype,
                                        acc_dtype=acc_dtype)
            self.shards.append(sh)

    def run_stage(self, rnd: int, stage: int) -> None:
        w = self.w
        counts = w.stage_counts(rnd, stage)
        for sh, (a, b) in zip(self.shards, self.slices):
            for wk in range(w.workers):
                for mb in range(counts[wk]):
                    sh.add_microbatch(wk, synth.host_grad_bf16(w.grad_spec(rnd, stage, wk, mb), a,
                                                               b - a))
            if stage == synth.STAGE_TILDE:
                sh.stage1()
            else:
                sh.stage2()


# ------------------------------------------------------------------ GPU runs


def gpu_run_stage(owner, w: synth.Workload, rnd: int, stage: int, grad_buf,
                  fresh_buffers: bool = False) -> None:
    """Feed one stage of round rnd through the HIP library (full shard, device-generated).
    fresh_buffers: every micro-batch gradient gets a buffer of its own (instead of one buffer
    that the next micro-batch overwrites), as an owner that adopts buffers needs."""
    import torch
    counts = w.stage_counts(rnd, stage)
    for wk in range(w.workers):
        for mb in range(counts[wk]):
            if fresh_buffers:
                grad_buf = torch.empty_like(grad_buf)
            synth.device_grad_bf16(grad_buf, w.grad_spec(rnd, stage, wk, mb), 0)
            owner.add_microbatch(wk, grad_buf, last=(mb == counts[wk] - 1))
    if stage == synth.STAGE_TILDE:
        owner.stage1()
    else:
        owner.stage2()


def gather(t, slices):
    """Host copy of the listed index ranges of a device tensor, concatenated."""
    import torch
    parts = [t[a:b] for a, b in slices]
    return torch.cat(parts).cpu()
