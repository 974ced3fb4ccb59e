"""Pins for the oracle's AdamW element update, estimate and commit.

Closed forms, exact rational arithmetic and torch's CPU AdamW; nothing here
re-types the oracle's own formula as the expected value.
"""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

PREC = ["f64", "f32"]
TOL_REL, TOL_ABS = 2e-6, 1e-9


def close(a, b, rel=TOL_REL, abs_=TOL_ABS):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.all((np.abs(a - b) <= abs_) | (np.abs(a - b) <= rel * np.abs(b)))


def ulp_diff(a, b):
    a = np.asarray(a, np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, np.float32).view(np.int32).astype(np.int64)
    a = np.where(a < 0, np.int64(-2 ** 31) - a, a)
    b = np.where(b < 0, np.int64(-2 ** 31) - b, b)
    return np.abs(a - b)


def hyper(lr=6e-4, b1=0.9, b2=0.95, eps=1e-8, wd=0.1):
    return oracle.make_hyper(lr, b1, b2, eps, wd)


# ------------------------------------------------------------------ closed forms


@pytest.mark.parametrize("precision", PREC)
@pytest.mark.parametrize("eps", [1e-8, 1e-3])
def test_first_step_is_lr_g_over_abs_g_plus_eps(precision, eps):
    # step 1 from m = v = 0 with no decay: m^ = g, v^ = g^2, so dtheta = -lr g / (|g| + eps).
    rng = np.random.default_rng(0)
    n = 50_000
    g = (rng.standard_normal(n) * np.exp(rng.uniform(-12, 0, n))).astype(np.float32)
    theta0 = rng.uniform(-0.05, 0.05, n).astype(np.float32)
    theta, m, v = theta0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    lr = 6e-4
    oracle.commit(theta, m, v, g, hyper(lr=lr, eps=eps, wd=0.0), step=1, count=1,
                  precision=precision)
    gd = g.astype(np.float64)
    want = theta0.astype(np.float64) - lr * gd / (np.abs(gd) + eps)
    assert close(theta, want)
    # the update itself, not just theta, is right: compare the step to 1e-5 of lr
    assert np.all(np.abs((theta.astype(np.float64) - theta0) - (want - theta0)) <= 1e-5 * lr + 4e-9)
    assert close(m, 0.1 * gd) and close(v, 0.05 * gd * gd, abs_=1e-30)


@pytest.mark.parametrize("precision", PREC)
def test_first_step_scales_gradient_sum_by_count(precision):
    # gsum / count is what enters the moments: m' = (1-b1) gsum/count, v' = (1-b2) (gsum/count)^2
    rng = np.random.default_rng(1)
    n = 10_000
    gsum = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    for count in (1, 2, 3, 7, 32, 37):
        theta, m, v = np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32)
        oracle.commit(theta, m, v, gsum, hyper(wd=0.0), step=1, count=count, precision=precision)
        g = gsum.astype(np.float64) / count
        assert close(m, 0.1 * g) and close(v, 0.05 * g * g, abs_=1e-30)


@pytest.mark.parametrize("precision", PREC)
def test_zero_learning_rate_leaves_theta_bitwise_unchanged(precision):
    rng = np.random.default_rng(2)
    n = 20_000
    theta0 = rng.standard_normal(n).astype(np.float32)
    theta = theta0.copy()
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (rng.random(n) * 1e-6).astype(np.float32)
    m0, v0 = m.copy(), v.copy()
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    oracle.commit(theta, m, v, g, hyper(lr=0.0), step=5, count=1, precision=precision)
    assert np.array_equal(theta.view(np.uint32), theta0.view(np.uint32))
    # the moments still move
    assert close(m, 0.9 * m0.astype(np.float64) + 0.1 * g.astype(np.float64))
    assert close(v, 0.95 * v0.astype(np.float64) + 0.05 * g.astype(np.float64) ** 2, abs_=1e-30)


@pytest.mark.parametrize("precision", PREC)
def test_zero_gradient_is_pure_decoupled_decay(precision):
    rng = np.random.default_rng(3)
    n = 20_000
    theta0 = rng.standard_normal(n).astype(np.float32)
    theta, m, v = theta0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    lr, wd = 6e-4, 0.1
    oracle.commit(theta, m, v, np.zeros(n, np.float32), hyper(lr=lr, wd=wd), step=1, count=4,
                  precision=precision)
    want = (theta0.astype(np.float64) * (1.0 - lr * wd)).astype(np.float32)
    assert ulp_diff(theta, want).max() <= 1
    assert not m.any() and not v.any()
    # and it is decay of theta, not an L2 term pushed through Adam's normalisation
    # (that would move every theta by about lr, independent of its size)
    assert np.max(np.abs(theta - theta0)) < lr * wd * np.max(np.abs(theta0)) * 1.001


@pytest.mark.parametrize("precision", PREC)
def test_constant_gradient_many_steps(precision):
    # constant g: m_t = g (1 - b1^t), v_t = g^2 (1 - b2^t) => every step moves theta by
    # -lr g/(|g|+eps) when there is no decay.
    n, T, lr, eps = 4096, 60, 1e-3, 1e-8
    rng = np.random.default_rng(4)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    theta0 = rng.uniform(-1, 1, n).astype(np.float32)
    theta, m, v = theta0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    hp = hyper(lr=lr, eps=eps, wd=0.0)
    for t in range(1, T + 1):
        oracle.commit(theta, m, v, g, hp, step=t, count=1, precision=precision)
    gd = g.astype(np.float64)
    assert close(m, gd * (1 - 0.9 ** T), rel=1e-5)
    assert close(v, gd * gd * (1 - 0.95 ** T), rel=1e-5, abs_=1e-30)
    want = theta0.astype(np.float64) - T * lr * gd / (np.abs(gd) + eps)
    # theta is stored in fp32 after every step: up to half an ulp of rounding per step
    store = T * 2.0 ** -24 * np.maximum(np.abs(theta0), np.abs(want))
    assert np.all(np.abs(theta - want) <= 1e-5 * T * lr + store)


# ------------------------------------------------------------------ exact arithmetic


def _exact_update(theta, m, v, gsum, count, lr, b1, b2, eps, wd, step):
    """AdamW (decoupled decay, bias-corrected, eps outside the root) in exact rationals;
    the square root to 50 digits."""
    getcontext().prec = 60
    F = Fraction
    g = F(float(gsum)) / count
    m1 = F(b1) * F(float(m)) + (1 - F(b1)) * g
    v1 = F(b2) * F(float(v)) + (1 - F(b2)) * g * g
    mh = m1 / (1 - F(b1) ** step)
    vh = v1 / (1 - F(b2) ** step)
    root = (Decimal(vh.numerator) / Decimal(vh.denominator)).sqrt()
    root = F(root)
    th = F(float(theta))
    t1 = th - F(lr) * F(wd) * th - F(lr) * mh / (root + F(eps))
    return float(t1), float(m1), float(v1)


@pytest.mark.parametrize("precision,max_ulp", [("f64", 1), ("f32", 4)])
def test_against_exact_rational_arithmetic(precision, max_ulp):
    rng = np.random.default_rng(5)
    n = 300
    lr, b1, b2, eps, wd = 6e-4, 0.9, 0.95, 1e-8, 0.1
    for step, count in ((1, 1), (2, 3), (17, 8), (1000, 37)):
        theta = rng.standard_normal(n).astype(np.float32) * np.float32(0.02)
        m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
        v = (rng.random(n) * 1e-8).astype(np.float32)
        gsum = (rng.standard_normal(n) * 1e-3 * count).astype(np.float32)
        want = [_exact_update(theta[i], m[i], v[i], gsum[i], count, lr, b1, b2, eps, wd, step)
                for i in range(n)]
        wt, wm, wv = (np.array(c, np.float64) for c in zip(*want))
        th0 = theta.astype(np.float64)
        oracle.commit(theta, m, v, gsum, hyper(lr, b1, b2, eps, wd), step=step, count=count,
                      precision=precision)
        if precision == "f64":
            assert ulp_diff(theta, wt.astype(np.float32)).max() <= max_ulp
        else:
            # binary32 arithmetic: rounding of m' (which may cancel) is amplified by
            # step_size/den, so the bound is the path's stated tolerance, not a few ulp
            assert close(theta, wt)
            scale = np.maximum(np.maximum(np.abs(wt), np.abs(th0)), np.abs(wt - th0))
            assert np.median(np.abs(theta - wt) / (2.0 ** -24 * scale)) <= 1.0
        # m can cancel (b1 m and (1-b1) g of opposite sign): bound the error by the terms' size
        assert close(m, wm, rel=1e-6, abs_=1e-10)
        assert ulp_diff(v, wv.astype(np.float32)).max() <= max_ulp


def test_pins_tell_common_mistakes_apart():
    """The inputs used above separate AdamW from its usual mis-implementations by far more
    than the tolerance, so a pin that passes does mean something."""
    rng = np.random.default_rng(6)
    n = 1000
    lr, b1, b2, eps, wd, step = 6e-4, 0.9, 0.95, 1e-3, 0.1, 3
    theta = rng.standard_normal(n) * 0.5
    m = rng.standard_normal(n) * 1e-3
    v = rng.random(n) * 1e-6
    g = rng.standard_normal(n) * 1e-3
    m1, v1 = b1 * m + (1 - b1) * g, b2 * v + (1 - b2) * g * g
    bc1, bc2 = 1 - b1 ** step, 1 - b2 ** step
    right = theta * (1 - lr * wd) - lr * (m1 / bc1) / (np.sqrt(v1 / bc2) + eps)
    mutants = {
        "eps inside root": theta * (1 - lr * wd) - lr * (m1 / bc1) / np.sqrt(v1 / bc2 + eps),
        "eps before bias correction": theta * (1 - lr * wd)
        - lr * (m1 / bc1) / ((np.sqrt(v1) + eps) / np.sqrt(bc2)),
        "no bias correction": theta * (1 - lr * wd) - lr * m1 / (np.sqrt(v1) + eps),
        "coupled L2": theta - lr * ((b1 * m + (1 - b1) * (g + wd * theta)) / bc1)
        / (np.sqrt((b2 * v + (1 - b2) * (g + wd * theta) ** 2) / bc2) + eps),
        "sign": theta * (1 - lr * wd) + lr * (m1 / bc1) / (np.sqrt(v1 / bc2) + eps),
        "betas swapped": theta * (1 - lr * wd)
        - lr * ((b2 * m + (1 - b2) * g) / bc1) / (np.sqrt((b1 * v + (1 - b1) * g * g) / bc2) + eps),
    }
    th32 = theta.astype(np.float32)
    got = th32.copy()
    mm, vv = m.astype(np.float32), v.astype(np.float32)
    oracle.commit(got, mm, vv, g.astype(np.float32), hyper(lr, b1, b2, eps, wd), step, 1)
    assert np.max(np.abs(got - right)) < 2e-7
    for name, wrong in mutants.items():
        assert np.median(np.abs(wrong - right)) > 1e-5, name


# ------------------------------------------------------------------ library special case


@pytest.mark.parametrize("precision", PREC)
@pytest.mark.parametrize("wd,lr,eps", [(0.1, 6e-4, 1e-8), (0.0, 2e-5, 1e-8), (0.05, 1e-2, 1e-4)])
def test_commit_only_sequence_is_plain_adamw_as_torch_cpu_computes_it(precision, wd, lr, eps):
    # eq. (DDP): theta(t+1) = Opt(theta(t), normalised batch gradient).  torch.optim.AdamW on the
    # CPU in fp32 (single-tensor path) is that Opt.
    torch.manual_seed(0)
    n, T = 20_000, 25
    p = torch.nn.Parameter((torch.randn(n) * 0.02).float())
    opt = torch.optim.AdamW([p], lr=lr, betas=(0.9, 0.95), eps=eps, weight_decay=wd,
                            foreach=False, fused=False, amsgrad=False)
    theta = p.detach().numpy().copy()
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    hp = hyper(lr, 0.9, 0.95, eps, wd)
    for t in range(1, T + 1):
        g = (torch.randn(n) * 1e-3).float()
        p.grad = g.clone()
        opt.step()
        oracle.commit(theta, m, v, g.numpy(), hp, step=t, count=1, precision=precision)
    st = opt.state[p]
    # torch multiplies theta by fp32(1 - lr wd) each step, a factor that is off by up to
    # 2^-25 relative: allow for that drift on top of the path's tolerance
    drift = T * 2.0 ** -25
    assert close(theta, p.detach().numpy(), rel=TOL_REL + drift, abs_=TOL_ABS + drift * 0.1)
    assert close(m, st["exp_avg"].numpy())
    assert close(v, st["exp_avg_sq"].numpy(), abs_=1e-30)


# ------------------------------------------------------------------ estimate


@pytest.mark.parametrize("precision", PREC)
def test_estimate_reads_only_and_equals_what_commit_would_write(precision):
    rng = np.random.default_rng(8)
    n = 30_001
    theta = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    v = (rng.random(n) * 1e-8).astype(np.float32)
    g = (rng.standard_normal(n) * 4e-4).astype(np.float32)
    keep = [a.copy() for a in (theta, m, v, g)]
    hp = hyper()
    t_f32, t_bf16 = oracle.estimate(theta, m, v, g, hp, step=7, count=4, precision=precision)
    for a, b in zip((theta, m, v, g), keep):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    c_bf16 = oracle.commit(theta, m, v, g, hp, step=7, count=4, precision=precision)
    assert np.array_equal(t_f32.view(np.uint32), theta.view(np.uint32))
    assert np.array_equal(t_bf16, c_bf16)
    # the bf16 output is the RNE cast of the fp32 one (torch as the independent cast)
    want = torch.from_numpy(t_f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(t_bf16, want)
    # outputs are optional one at a time
    only32, none16 = oracle.estimate(keep[0], keep[1], keep[2], g, hp, 7, 4, want_bf16=False,
                                     precision=precision)
    assert none16 is None and np.array_equal(only32, t_f32)


def test_f32_form_stays_within_tolerance_of_f64_form_over_many_rounds():
    rng = np.random.default_rng(9)
    n, T = 50_000, 50
    th64 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    th32 = th64.copy()
    th0 = th64.astype(np.float64)
    m64, v64, m32, v32 = (np.zeros(n, np.float32) for _ in range(4))
    hp = hyper()
    for t in range(1, T + 1):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        oracle.commit(th64, m64, v64, g, hp, t, 8, precision="f64")
        oracle.commit(th32, m32, v32, g, hp, t, 8, precision="f32")
        if t == 10:
            err10, ref10 = np.abs(th32.astype(np.float64) - th64), th64.astype(np.float64)
    # two correct implementations differ by independent roundings of about an ulp of the
    # LARGEST magnitude theta took along the way, so the relative bound uses that magnitude
    err = np.abs(th32.astype(np.float64) - th64)
    # and the absolute floor grows with the number of Adam steps of size ~lr that were summed
    assert np.all((err <= TOL_ABS * T / 10)
                  | (err <= TOL_REL * np.maximum(np.abs(th64), np.abs(th0))))
    assert close(m32, m64) and close(v32, v64, abs_=1e-30)
    # after the ten rounds of the longest workload all but a handful of elements meet the
    # plain per-element tolerance as well
    assert np.mean((err10 > TOL_ABS) & (err10 > TOL_REL * np.abs(ref10))) < 1e-4
