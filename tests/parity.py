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


# ------------------------------------------------------------------ optimizer states

U32 = 2.0 ** -24                       # unit roundoff of binary32, round to nearest


def adam_state(rng, n: int, kind: str, hyper=None, step: int = 1, count: int = 1, gsum=None):
    """(theta, m, v, gsum) for the step entry points.  `step` is the index of the update the
    state is meant for (1-based), `count` its micro-batch count; a given `gsum` is used as it is.

    cold   m = v = 0 (the first update);
    warm   a state Adam can be in after many similar steps: |m| / sqrt(v) of order one, so
           every step is of order lr and theta' stays of theta's magnitude;
    wide   nothing assumed about how m and v got there.  Thirds of the array:
           (a) m ~ N(0, 1e-4) against v ~ U(0, 1e-8), independent of each other;
           (b) |m| / sqrt(v) log-uniform in [1, 1e3] (steps up to 1e3 lr, far larger than theta);
           (c) v zero, denormal or tiny with m non-zero, so that eps or the gradient of this
               very step decides the denominator;
           and, on every 5th element when `hyper` is given, theta chosen so that the decayed
           theta and the Adam step cancel (theta' is a rounding residue of two numbers of
           theta's size).
    Special lanes (exact zeros in gsum, a gradient whose square underflows, a denormal v,
    +0 / -0 in theta) are planted in every kind when n > 16.
    """
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    given = gsum is not None
    if not given:
        gsum = (rng.standard_normal(n) * 4e-4).astype(np.float32)
        if n > 16:
            gsum[::7] = 0.0                      # exact zeros: the pure-decay path
            gsum[3] = 1e-30                      # g^2 underflows to a denormal / zero
    if kind == "cold":
        m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    elif kind == "warm":
        m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
        v = (m.astype(np.float64) ** 2 * rng.uniform(0.5, 4.0, n) + 1e-12 * rng.random(n)).astype(
            np.float32)
    elif kind == "wide":
        m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
        v = rng.uniform(0.0, 1e-8, n).astype(np.float32)
        third = n // 3
        ratio = 10.0 ** rng.uniform(0.0, 3.0, third)
        v[third:2 * third] = ((m[third:2 * third].astype(np.float64) / ratio) ** 2).astype(np.float32)
        tail = n - 2 * third
        tiny = np.array([0.0, 1e-45, 1e-42, 1e-39, 1.2e-38, 1e-30, 1e-20], np.float32)
        v[2 * third:] = tiny[rng.integers(0, tiny.size, tail)]
        if hyper is not None and n > 16:
            # theta (1 - lr wd) = lr/(1-b1^t) m' / (sqrt(v')/sqrt(1-b2^t) + eps), in binary64
            lr, b1, b2, eps, wd = (hyper[k] for k in ("lr", "b1", "b2", "eps", "wd"))
            if lr > 0 and lr * wd < 1:
                g = gsum.astype(np.float64) / count
                m1 = b1 * m.astype(np.float64) + (1 - b1) * g
                v1 = b2 * v.astype(np.float64) + (1 - b2) * g * g
                a = lr / (1 - b1 ** step) * m1 / (np.sqrt(v1) / np.sqrt(1 - b2 ** step) + eps)
                with np.errstate(over="ignore", invalid="ignore"):
                    cancel = (a / (1 - lr * wd)).astype(np.float32)
                ok = np.isfinite(cancel)
                ok[np.arange(n) % 5 != 0] = False
                theta[ok] = cancel[ok]
    else:
        raise ValueError(kind)
    if n > 16:
        v[5] = 1e-42                             # denormal second moment
        theta[9] = 0.0
        theta[11] = -0.0
    return theta, m, v, gsum


def theta_bound(theta, m, v, gsum, hyper, step: int, count: int) -> np.ndarray:
    """Per-element bound on |theta'_binary32 - theta'_binary64| for one AdamW update.

    With u = 2^-24, T = theta (1 - lr wd) and the Adam step A = lr/(1-b1^t) m'/den: the
    binary32 form makes at most 5u S relative-to-S error in m' where S = b1 |m| + (1-b1) |g|
    (S, not |m'|: the two terms may cancel), 8u in den (all its terms are non-negative), so
    14u A_abs in the product with the rounded step size, A_abs = lr/(1-b1^t) S / den; the
    decayed theta and the final fused operation add (2 + lr wd) u |theta| + u A_abs, and the
    binary64 form's one rounding to fp32 another u (|theta| + A_abs).  Altogether
        |d theta'| <= 16 u (|theta| + A_abs)   (for lr wd <= 10),
    which is below 2e-6 max(|theta|, A_abs).  The floor covers results in the denormal range.
    """
    lr, b1, b2, eps, wd = (hyper[k] for k in ("lr", "b1", "b2", "eps", "wd"))
    g = gsum.astype(np.float64) / count
    s = b1 * np.abs(m.astype(np.float64)) + (1 - b1) * np.abs(g)
    v1 = b2 * v.astype(np.float64) + (1 - b2) * g * g
    with np.errstate(divide="ignore", invalid="ignore"):
        a_abs = lr / (1 - b1 ** step) * s / (np.sqrt(v1) / np.sqrt(1 - b2 ** step) + eps)
    a_abs = np.nan_to_num(a_abs, nan=0.0, posinf=np.finfo(np.float64).max / 1e6)
    return 16 * U32 * (np.abs(theta.astype(np.float64)) + a_abs) + 2.0 ** -140


def assert_theta_within_bound(got, want64, bound, what=""):
    g, w = got.astype(np.float64), want64.astype(np.float64)
    both_nan = np.isnan(g) & np.isnan(w)
    with np.errstate(invalid="ignore"):
        err = np.where(both_nan | (g == w), 0.0, np.abs(g - w))
    bad = ~(err <= bound)
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} beyond the derived bound; first "
                           f"at {int(np.argmax(bad))}: got {got[np.argmax(bad)]!r} want "
                           f"{want64[np.argmax(bad)]!r} bound {bound[np.argmax(bad)]!r}")


def assert_bf16_within_bound(got_bits, want_bits, want_f32, bound, what=""):
    """bf16 outputs against the binary64 form when the fp32 values underneath are only known to
    agree within `bound`: where the bound is below one bf16 ulp of the value (2^-8 |x|), the two
    roundings can differ by at most one ulp; elsewhere (theta' a residue of a cancellation) the
    bf16 values can differ by the bound plus the two roundings."""
    both_nan = ((got_bits & 0x7FFF) > 0x7F80) & ((want_bits & 0x7FFF) > 0x7F80)
    d = np.where(both_nan, 0, bf16_ulp_distance(got_bits, want_bits))
    gv = oracle.bf16_to_f32(np.ascontiguousarray(got_bits)).astype(np.float64)
    wv = oracle.bf16_to_f32(np.ascontiguousarray(want_bits)).astype(np.float64)
    x = np.abs(want_f32.astype(np.float64))
    strict = bound <= 2.0 ** -8 * x
    with np.errstate(invalid="ignore"):
        loose_ok = np.abs(gv - wv) <= bound + 2.0 ** -8 * (np.abs(gv) + np.abs(wv))
    bad = np.where(strict, d > BF16_MAX_ULP, ~(loose_ok | both_nan | (d == 0)))
    assert not bad.any(), (f"{what}: bf16 differs at {int(np.argmax(bad))}: "
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
    that the next micro-batch overwrites), as an owner that adopts buffers needs.
    A batched owner gets the k-th micro-batch of all workers at once (one buffer per worker)."""
    import torch
    counts = w.stage_counts(rnd, stage)
    if owner.batched:
        if not hasattr(owner, "_parity_bufs"):
            owner._parity_bufs = [grad_buf] + [torch.empty_like(grad_buf)
                                               for _ in range(w.workers - 1)]
        for mb in range(max(counts)):
            items = []
            for wk in range(w.workers):
                if mb < counts[wk]:
                    buf = torch.empty_like(grad_buf) if fresh_buffers else owner._parity_bufs[wk]
                    synth.device_grad_bf16(buf, w.grad_spec(rnd, stage, wk, mb), 0)
                    items.append((wk, buf, mb == counts[wk] - 1))
            owner.add_microbatches(items)
    else:
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
