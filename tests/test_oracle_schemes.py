"""Pins for the oracle's SGD step and for the sequencing of the four update schemes
(eq. DDP, DPU, WP, ACCO): on f(x) = a x^2 / 2 per coordinate every scheme with Opt = GD is a
linear recursion with a closed form (matrix powers), among them the recursion of the paper's
Prop. GD for ACCO."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle.schemes import OracleScheme


def quad_setup(n=257, seed=0):
    rng = np.random.default_rng(seed)
    a = rng.uniform(0.2, 2.0, n)                       # curvatures, L = 2
    x0 = rng.standard_normal(n)
    return a.astype(np.float32), x0.astype(np.float32)


def closed_form(scheme, a, x0, eta, T, xt0=None):
    """(theta_T, params_T) in float64 by explicit 2x2 matrix powers per coordinate."""
    a = a.astype(np.float64)
    th = x0.astype(np.float64)
    tt = th.copy() if xt0 is None else xt0.astype(np.float64)
    out_t, out_p = np.empty_like(th), np.empty_like(th)
    for k in range(a.size):
        ea = eta * a[k]
        if scheme == "acco":     # Prop. GD: state (theta, theta~)
            M = np.array([[1 - ea / 2, -ea / 2], [1.0, -ea]])
            s = np.linalg.matrix_power(M, T) @ np.array([th[k], tt[k]])
            out_t[k], out_p[k] = s[0], s[0]            # after a full round the buffer holds theta
        elif scheme == "ddp":
            out_t[k] = out_p[k] = (1 - ea) ** T * th[k]
        elif scheme == "dpu":    # theta_{t+1} = theta_t - ea theta_{t-1}, first step undelayed
            M = np.array([[1.0, -ea], [1.0, 0.0]])     # state (theta_t, theta_{t-1})
            s = np.array([(1 - ea) * th[k], th[k]])    # after round 0
            s = np.linalg.matrix_power(M, T - 1) @ s
            out_t[k], out_p[k] = s[0], s[1]            # compute uses theta(t-1)
        else:                    # wp: state (theta, theta~)
            M = np.array([[1.0, -ea], [1.0, -2 * ea]])
            s = np.linalg.matrix_power(M, T) @ np.array([th[k], tt[k]])
            out_t[k], out_p[k] = s[0], s[1]
    return out_t, out_p


def run_quadratic(owner, scheme, a, T, grad_of, xt0=None):
    """Drive a scheme with gradients a * (parameters the compute stream holds)."""
    if scheme == "acco":
        g_half = grad_of(owner.params if xt0 is None else xt0)   # g~_0 at theta~_0
        g_full = grad_of(owner.params)                           # g_0 at theta_0
        for _ in range(T):
            owner.set_gradient_f32(0, g_half, 1)
            owner.finish_half()
            g_half = grad_of(owner.params)                       # g~_{t+1} at theta~_{t+1}
            owner.set_gradient_f32(0, g_full, 1)
            owner.finish_round()
            g_full = grad_of(owner.params)                       # g_{t+1} at theta_{t+1}
    else:
        g = grad_of(owner.params)
        for _ in range(T):
            owner.set_gradient_f32(0, g, 1)
            owner.finish_round()
            g = grad_of(owner.params)


@pytest.mark.parametrize("precision", ["f64", "f32"])
@pytest.mark.parametrize("scheme", ["acco", "ddp", "dpu", "wp"])
def test_gd_on_a_quadratic_follows_the_closed_form_recursion(scheme, precision):
    a, x0 = quad_setup()
    eta, T = 0.2, 25                                   # eta <= 1/(2L) as Prop. GD asks
    o = OracleScheme(x0, 1, scheme, sgd_lr=eta, comm_dtype="f32", precision=precision)
    run_quadratic(o, scheme, a, T, lambda p: (a * p).astype(np.float32))
    want_t, want_p = closed_form(scheme, a, x0, eta, T)
    scale = np.abs(x0).max()
    assert np.max(np.abs(o.theta - want_t)) <= 2e-6 * scale
    assert np.max(np.abs(o.params - want_p)) <= 2e-6 * scale
    assert o.step == T
    # the schemes really differ from one another on this problem
    # (compared after 3 rounds, before everything has decayed to the minimiser)
    mine = closed_form(scheme, a, x0, eta, 3)[0]
    # acco and ddp coincide here: with exact gradients and theta~_0 = theta_0 the estimate
    # equals the commit, which is the sense in which ACCO 'does not rely on an approximation';
    # the next test separates them with theta~_0 != theta_0
    same = {"acco": "ddp", "ddp": "acco"}.get(scheme)
    others = [closed_form(s, a, x0, eta, 3)[0] for s in ("acco", "ddp", "dpu", "wp")
              if s not in (scheme, same)]
    assert all(np.max(np.abs(w - mine)) > 1e-3 * scale for w in others)


def dpu_warm_closed_form(a, x0, eta, T, warm):
    """DPU after `warm` undelayed rounds: plain GD for `warm` rounds, then the first delayed round
    still differentiates the parameters the last undelayed round handed out, and from there on
    theta_{t+1} = theta_t - eta a theta_{t-1}."""
    a = a.astype(np.float64)
    out_t, out_p = np.empty(a.size), np.empty(a.size)
    for k in range(a.size):
        ea = eta * a[k]
        th = (1 - ea) ** min(warm, T) * float(x0[k])
        if T <= warm:
            out_t[k] = out_p[k] = th
            continue
        s = np.array([(1 - ea) * th, th])              # after the first delayed round
        s = np.linalg.matrix_power(np.array([[1.0, -ea], [1.0, 0.0]]), T - warm - 1) @ s
        out_t[k], out_p[k] = s[0], s[1]
    return out_t, out_p


@pytest.mark.parametrize("warm", [0, 1, 5, 30])
def test_dpu_with_undelayed_warm_up_rounds_follows_its_closed_form(warm):
    a, x0 = quad_setup(seed=6)
    eta, T = 0.2, 25
    o = OracleScheme(x0, 1, "dpu", sgd_lr=eta, comm_dtype="f32", warmup_rounds=warm)
    run_quadratic(o, "dpu", a, T, lambda p: (a * p).astype(np.float32))
    want_t, want_p = dpu_warm_closed_form(a, x0, eta, T, warm)
    scale = np.abs(x0).max()
    assert np.max(np.abs(o.theta - want_t)) <= 2e-6 * scale
    assert np.max(np.abs(o.params - want_p)) <= 2e-6 * scale
    # no warm-up is the plain scheme; warm-up past the horizon is DDP
    if warm == 0:
        assert np.allclose(want_t, closed_form("dpu", a, x0, eta, T)[0], rtol=0, atol=1e-12)
    if warm >= T:
        assert np.allclose(want_t, closed_form("ddp", a, x0, eta, T)[0], rtol=0, atol=1e-12)
    else:
        assert np.max(np.abs(want_t - closed_form("ddp", a, x0, eta, T)[0])) > 1e-6 * scale


def test_acco_gd_with_distinct_initial_estimate_and_the_propositions_bound():
    # Prop. GD allows theta~_0 != theta_0; its bound on the summed squared gradient norms holds
    a, x0 = quad_setup(seed=3)
    rng = np.random.default_rng(4)
    xt0 = (x0 + 0.3 * rng.standard_normal(x0.size)).astype(np.float32)
    eta, T, L = 0.25, 40, 2.0
    o = OracleScheme(x0, 1, "acco", sgd_lr=eta, comm_dtype="f32")
    f = lambda x: 0.5 * np.sum(a.astype(np.float64) * x.astype(np.float64) ** 2)
    lhs = 0.0
    th, tt = x0.copy(), xt0.copy()
    g_half, g_full = (a * tt).astype(np.float32), (a * th).astype(np.float32)
    for _ in range(T):
        lhs += np.sum((a * th).astype(np.float64) ** 2) + np.sum((a * tt).astype(np.float64) ** 2)
        o.set_gradient_f32(0, g_half, 1)
        o.finish_half()
        tt = o.params.copy()
        g_half = (a * tt).astype(np.float32)
        o.set_gradient_f32(0, g_full, 1)
        o.finish_round()
        th = o.params.copy()
        g_full = (a * th).astype(np.float32)
    want_t, _ = closed_form("acco", a, x0, eta, T, xt0)
    assert np.max(np.abs(o.theta - want_t)) <= 2e-6 * np.abs(x0).max()
    rhs = 8.0 / (eta * T) * (f(x0) + f(xt0) + L * np.sum((x0.astype(np.float64) - xt0) ** 2))
    assert lhs / T <= rhs


@pytest.mark.parametrize("precision,ulps", [("f64", 0.5), ("f32", 1.5)])
def test_sgd_step_against_exact_rationals(precision, ulps):
    rng = np.random.default_rng(5)
    n = 400
    theta = rng.standard_normal(n).astype(np.float32)
    gsum = (rng.standard_normal(n) * 3).astype(np.float32)
    lr, wd = 0.05, 0.1
    for count in (1, 3, 8):
        got, bits = oracle.sgd_step(theta, gsum, lr, wd, count, commit=False, precision=precision)
        want = np.array([float(Fraction(float(t)) * (1 - Fraction(lr) * Fraction(wd))
                               - Fraction(lr) * Fraction(float(g)) / count)
                         for t, g in zip(theta, gsum)])
        ulp = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
        scale = np.maximum(ulp, np.spacing(np.abs(theta)).astype(np.float64))
        assert np.all(np.abs(got - want) <= ulps * scale * 1.001)
        assert np.array_equal(bits, oracle.cast(got))
    # commit writes in place what estimate returns; lr = 0 is the identity; g = 0 pure decay
    t2 = theta.copy()
    oracle.sgd_step(t2, gsum, lr, wd, 8, commit=True, want_bf16=False, precision=precision)
    assert np.array_equal(t2, got)
    t3 = theta.copy()
    oracle.sgd_step(t3, gsum, 0.0, wd, 8, commit=True, want_bf16=False, precision=precision)
    assert np.array_equal(t3.view(np.uint32), theta.view(np.uint32))


def test_adamw_schemes_reduce_to_their_definitions():
    # one round from a common state with synthetic gradients: ddp/dpu/wp commit the same theta;
    # dpu hands out the old theta, ddp the new one, wp one more speculative step on the same g
    import synth
    w = synth.Workload(name="s", n=3000, workers=2, rounds=1, grad_std=1e-3, k_fixed=2, seed=9)
    hp = oracle.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    th0 = w.host_theta(0, w.n)
    res = {}
    for scheme in ("ddp", "dpu", "wp"):
        o = OracleScheme(th0, w.workers, scheme, adamw=hp, precision="f32")
        for wk in range(w.workers):
            for st in (1, 2):
                o.add_microbatch(wk, synth.host_grad_bf16(w.grad_spec(0, st, wk, 0), 0, w.n))
        o.finish_round()
        res[scheme] = o
    for s in ("dpu", "wp"):
        assert np.array_equal(res[s].theta.view(np.uint32), res["ddp"].theta.view(np.uint32))
    assert np.array_equal(res["ddp"].params, res["ddp"].theta)
    assert np.array_equal(res["dpu"].params, th0)
    o = res["wp"]
    want, _ = oracle.estimate(o.theta, o.m, o.v, o.gsum, hp, 2, 4, precision="f32")
    assert np.array_equal(o.params.view(np.uint32), want.view(np.uint32))
    assert all(r.step == 1 and r.total == 4 for r in res.values())
