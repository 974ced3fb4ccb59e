"""The tolerance the GPU tests use on optimizer states that Adam itself need not have produced
(`parity.adam_state(kind="wide")`), checked on the CPU between the oracle's two forms.

The plain tolerance of the task (2e-6 relative or 1e-9 absolute) cannot hold for theta' where
the decayed theta and the Adam step cancel: both forms are correct to a few units in the last
place of the TERMS, not of the difference.  `parity.theta_bound` is the bound derived from the
binary32 operations; here it is shown to hold between the binary32 and the binary64 form, to be
needed (the plain tolerance fails on such states), and to be tight enough to tell a wrong
update from a right one.
"""
import numpy as np
import pytest

import oracle
from parity import (adam_state, assert_bf16_within_bound, assert_theta_within_bound, theta_bound)

HYPERS = [dict(lr=6e-4, b1=0.9, b2=0.95, eps=1e-8, wd=0.1),
          dict(lr=2e-5, b1=0.9, b2=0.95, eps=1e-8, wd=0.0),
          dict(lr=1e-2, b1=0.0, b2=0.5, eps=1e-3, wd=0.01),
          dict(lr=1e-3, b1=0.99, b2=0.999, eps=1e-12, wd=1.0)]
CASES = [(1, 1), (7, 32), (1001, 37), (100_000, 3)]


def ohp(h):
    return oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])


def both_forms(theta, m, v, gsum, h, step, count):
    out = {}
    for prec in ("f32", "f64"):
        t, mm, vv = theta.copy(), m.copy(), v.copy()
        b = oracle.commit(t, mm, vv, gsum, ohp(h), step, count, precision=prec)
        out[prec] = (t, mm, vv, b)
    return out


@pytest.mark.parametrize("hi", range(len(HYPERS)))
def test_binary32_form_is_within_the_derived_bound_of_the_binary64_form(hi):
    h = HYPERS[hi]
    rng = np.random.default_rng(100 + hi)
    n = 300_000
    worst, outside_plain = 0.0, 0
    for step, count in CASES:
        theta, m, v, gsum = adam_state(rng, n, "wide", h, step, count)
        r = both_forms(theta, m, v, gsum, h, step, count)
        bound = theta_bound(theta, m, v, gsum, h, step, count)
        t32, t64 = r["f32"][0], r["f64"][0]
        assert_theta_within_bound(t32, t64, bound)
        assert_bf16_within_bound(r["f32"][3], r["f64"][3], t64, bound)
        err = np.abs(t32.astype(np.float64) - t64)
        worst = max(worst, float((err / bound).max()))
        outside_plain += int(np.count_nonzero((err > 1e-9) & (err > 2e-6 * np.abs(t64))))
        # m and v have no cancellation at these magnitudes: the plain tolerance holds
        for k, abs_ in ((1, 1e-9), (2, 1e-30)):
            e = np.abs(r["f32"][k].astype(np.float64) - r["f64"][k])
            assert np.all((e <= abs_) | (e <= 2e-6 * np.abs(r["f64"][k])))
    # the bound is a worst case over ~16 roundings: what is seen uses a good part of it
    assert 0.05 < worst <= 1.0
    if h["lr"] >= 1e-4:
        assert outside_plain > 0          # which is why the plain tolerance is not the test


def test_the_bound_tells_a_wrong_update_from_a_right_one():
    """Mistakes planted in the oracle's inputs (never in the GPU code): each moves theta' far
    beyond the bound on most of the wide-state elements."""
    h = HYPERS[0]
    rng = np.random.default_rng(7)
    n, step, count = 100_000, 7, 32
    theta, m, v, gsum = adam_state(rng, n, "wide", h, step, count)
    bound = theta_bound(theta, m, v, gsum, h, step, count)
    right = both_forms(theta, m, v, gsum, h, step, count)["f64"][0].astype(np.float64)

    def frac_outside(hh, st, cnt):
        t, mm, vv = theta.copy(), m.copy(), v.copy()
        oracle.commit(t, mm, vv, gsum, ohp(hh), st, cnt, precision="f64")
        return float(np.mean(np.abs(t.astype(np.float64) - right) > bound))

    assert frac_outside(h, step, count) == 0.0
    assert frac_outside(dict(h, lr=h["lr"] * (1 + 1e-4)), step, count) > 0.5   # step size off by 1e-4
    assert frac_outside(h, step + 1, count) > 0.5                      # bias correction one step off
    assert frac_outside(h, step, count + 1) > 0.5                      # wrong normalisation
    assert frac_outside(dict(h, wd=0.0), step, count) > 0.5            # decay dropped
    assert frac_outside(dict(h, eps=1e-7), step, count) > 0.2          # epsilon ten times larger


def test_wide_states_are_what_they_claim():
    h = HYPERS[0]
    rng = np.random.default_rng(3)
    n = 90_000
    theta, m, v, gsum = adam_state(rng, n, "wide", h, 7, 32)
    third = n // 3
    with np.errstate(divide="ignore"):
        ratio = np.abs(m.astype(np.float64)) / np.sqrt(v.astype(np.float64))
    mid = ratio[third:2 * third]
    assert np.median(mid) > 10 and np.percentile(mid, 99) > 500          # up to 1e3
    tail = v[2 * third:]
    assert np.count_nonzero(tail == 0) > 100 and np.count_nonzero((tail > 0) & (tail < 1.2e-38)) > 100
    # the cancellation lanes: theta' is orders of magnitude below theta
    t64 = both_forms(theta, m, v, gsum, h, 7, 32)["f64"][0]
    lanes = np.arange(n) % 5 == 0
    lanes[[0, 5, 10]] = False
    big = np.abs(theta[lanes]) > 1e-6
    assert np.median(np.abs(t64[lanes][big]) / np.abs(theta[lanes][big])) < 1e-6
