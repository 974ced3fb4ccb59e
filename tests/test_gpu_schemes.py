"""SGD as Opt and the DDP / DPU / WP / ACCO sequencings on the GPU, against the oracle and
against the closed-form recursions (needs an MI355X)."""
import numpy as np
import pytest

import oracle
import synth
from oracle.schemes import OracleScheme
from parity import assert_f32_close, bit_mismatches, bits_of
from test_oracle_schemes import closed_form, quad_setup, run_quadratic

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def log(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def acco():
    import paper_2406_02613_amd as A
    assert torch.cuda.is_available()
    A.binding.lib()
    return A


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("shape", [(64, 1, 0), (128, 2, 1), (512, 4, 0)])
def test_sgd_steps_match_the_oracle(acco, shape):
    acco.set_launch_shape("sgd", *shape)
    rng = np.random.default_rng(20)
    for n in (0, 1, 5, 64, 1000, 4096 + 7, (1 << 20) + 37):
        for lr, wd, count in ((0.05, 0.0, 1), (6e-4, 0.1, 32), (0.0, 0.3, 3)):
            log("sgd", shape, n, lr, wd, count)
            theta = rng.standard_normal(n).astype(np.float32)
            gsum = (rng.standard_normal(n) * 2).astype(np.float32)
            td, gd = dev(theta), dev(gsum)
            o32 = torch.empty(n, dtype=torch.float32, device="cuda")
            o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            hp = acco.make_sgd(lr, wd)
            acco.acco_sgd_estimate_step(td, gd, hp, count, theta_tilde_f32=o32, theta_tilde_bf16=o16)
            assert bit_mismatches(td.cpu().numpy(), theta) == 0
            w32, w16 = oracle.sgd_step(theta, gsum, lr, wd, count, commit=False, precision="f32")
            w64, _ = oracle.sgd_step(theta, gsum, lr, wd, count, commit=False, precision="f64")
            assert bit_mismatches(o32.cpu().numpy(), w32) == 0
            assert np.array_equal(bits_of(o16), w16)
            # theta and lr*g are of order one here and may cancel: the absolute part of the
            # tolerance is a few ulp of the operands, not of the result
            assert_f32_close(o32.cpu().numpy(), w64, "sgd vs f64", abs_=5e-7)
            st = acco.Counter(4)
            c16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            acco.acco_sgd_commit_step(td, gd, hp, st, count, theta_bf16=c16)
            assert st.value == 5
            assert bit_mismatches(td.cpu().numpy(), w32) == 0
            assert np.array_equal(bits_of(c16), w16)
    acco.set_launch_shape("sgd", 64, 1, 0)


@pytest.mark.parametrize("scheme", ["acco", "ddp", "dpu", "wp"])
def test_gd_schemes_follow_the_closed_forms_and_the_oracle(acco, scheme):
    a, x0 = quad_setup(n=100_003, seed=1)
    eta, T = 0.2, 25
    ad = dev(a)
    g = acco.SchemeOwner(a.size, 1, scheme, acco.make_sgd(eta), comm_bf16=False)
    g.set_theta(dev(x0))
    o = OracleScheme(x0, 1, scheme, sgd_lr=eta, comm_dtype="f32", precision="f32")
    run_quadratic(g, scheme, a, T, lambda p: ad * p)
    run_quadratic(o, scheme, a, T, lambda p: (a * p).astype(np.float32))
    torch.cuda.synchronize()
    assert g.step.value == o.step == T
    assert bit_mismatches(g.theta.cpu().numpy(), o.theta) == 0
    assert bit_mismatches(g.params_f32.cpu().numpy(), o.params) == 0
    assert np.array_equal(bits_of(g.params_bf16), o.params_bf16)
    want_t, want_p = closed_form(scheme, a, x0, eta, T)
    scale = np.abs(x0).max()
    assert np.max(np.abs(g.theta.cpu().numpy() - want_t)) <= 2e-6 * scale
    assert np.max(np.abs(g.params_f32.cpu().numpy() - want_p)) <= 2e-6 * scale


@pytest.mark.parametrize("warm", [1, 4, 40])
def test_dpu_with_warm_up_rounds_matches_the_oracle_and_its_closed_form(acco, warm):
    from test_oracle_schemes import dpu_warm_closed_form
    a, x0 = quad_setup(n=60_007, seed=8)
    eta, T = 0.2, 12
    ad = dev(a)
    g = acco.SchemeOwner(a.size, 1, "dpu", acco.make_sgd(eta), comm_bf16=False, warmup_rounds=warm)
    g.set_theta(dev(x0))
    o = OracleScheme(x0, 1, "dpu", sgd_lr=eta, comm_dtype="f32", precision="f32",
                     warmup_rounds=warm)
    run_quadratic(g, "dpu", a, T, lambda p: ad * p)
    run_quadratic(o, "dpu", a, T, lambda p: (a * p).astype(np.float32))
    torch.cuda.synchronize()
    assert g.step.value == o.step == T
    assert bit_mismatches(g.theta.cpu().numpy(), o.theta) == 0
    assert bit_mismatches(g.params_f32.cpu().numpy(), o.params) == 0
    want_t, want_p = dpu_warm_closed_form(a, x0, eta, T, warm)
    scale = np.abs(x0).max()
    assert np.max(np.abs(g.theta.cpu().numpy() - want_t)) <= 2e-6 * scale
    assert np.max(np.abs(g.params_f32.cpu().numpy() - want_p)) <= 2e-6 * scale
    with pytest.raises(ValueError):
        acco.SchemeOwner(8, 1, "wp", acco.make_sgd(eta), warmup_rounds=2)


def test_acco_gd_with_distinct_initial_estimate(acco):
    a, x0 = quad_setup(n=50_001, seed=3)
    rng = np.random.default_rng(4)
    xt0 = (x0 + 0.3 * rng.standard_normal(x0.size)).astype(np.float32)
    eta, T = 0.25, 20
    ad = dev(a)
    g = acco.SchemeOwner(a.size, 1, "acco", acco.make_sgd(eta), comm_bf16=False)
    g.set_theta(dev(x0))
    run_quadratic(g, "acco", a, T, lambda p: ad * p, xt0=dev(xt0))
    want_t, _ = closed_form("acco", a, x0, eta, T, xt0)
    assert np.max(np.abs(g.theta.cpu().numpy() - want_t)) <= 2e-6 * np.abs(x0).max()


@pytest.mark.parametrize("scheme", ["acco", "ddp", "dpu", "wp"])
@pytest.mark.parametrize("comm_bf16", [True, False])
def test_adamw_schemes_match_the_oracle_on_synthetic_gradients(acco, scheme, comm_bf16):
    w = synth.Workload(name="sch", n=200_000 + 37, workers=3, rounds=3, grad_std=1e-3,
                       k_range=(2, 5), seed=13)
    h = w.hyper
    g = acco.SchemeOwner(w.n, w.workers, scheme,
                         acco.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                         comm_bf16=comm_bf16)
    th0 = w.host_theta(0, w.n)
    g.set_theta(dev(th0))
    refs = {p: OracleScheme(th0, w.workers, scheme,
                            adamw=oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                            comm_dtype="bf16" if comm_bf16 else "f32", precision=p)
            for p in ("f32", "f64")}
    buf = torch.empty(w.n, dtype=torch.bfloat16, device="cuda")
    for r in range(w.rounds):
        for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
            counts = w.stage_counts(r, stage)
            for wk in range(w.workers):
                for mb in range(counts[wk]):
                    sp = w.grad_spec(r, stage, wk, mb)
                    synth.device_grad_bf16(buf, sp, 0)
                    g.add_microbatch(wk, buf)
                    hb = synth.host_grad_bf16(sp, 0, w.n)
                    for o in refs.values():
                        o.add_microbatch(wk, hb)
            if stage == synth.STAGE_TILDE:
                if scheme == "acco":
                    g.finish_half()
                    for o in refs.values():
                        o.finish_half()
            else:
                g.finish_round()
                for o in refs.values():
                    o.finish_round()
            torch.cuda.synchronize()
        log("scheme", scheme, comm_bf16, "round", r)
        o = refs["f32"]
        assert g.step.value == o.step == r + 1
        assert g.total.value == o.total == sum(w.microbatches(r, k) for k in range(w.workers))
        for name in ("theta", "m", "v"):
            got = getattr(g, name).cpu().numpy()
            assert bit_mismatches(got, getattr(o, name)) == 0, name
            assert_f32_close(got, getattr(refs["f64"], name), f"{name} vs f64",
                             abs_=1e-30 if name == "v" else 1e-9 * (r + 1))
        assert bit_mismatches(g.params_f32.cpu().numpy(), o.params) == 0
        assert np.array_equal(bits_of(g.params_bf16), o.params_bf16)


@pytest.mark.parametrize("scheme", ["acco", "wp"])
def test_schemes_on_arena_placed_buffers_change_no_bits(acco, scheme):
    """The same rounds with every buffer of the scheme owner taken from an arena (state and
    communication buffers, accumulators and gradients, outputs by memory class)."""
    w = synth.Workload(name="sch_arena", n=150_000 + 5, workers=3, rounds=2, grad_std=1e-3,
                       k_range=(2, 4), seed=14)
    h = w.hyper
    arena = acco.HbmArena(2 << 30, step_bytes=512 << 20, probe_bytes=256 << 20)
    g = acco.SchemeOwner(w.n, w.workers, scheme,
                         acco.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                         arena=arena)
    th0 = w.host_theta(0, w.n)
    g.set_theta(dev(th0))
    o = OracleScheme(th0, w.workers, scheme,
                     adamw=oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                     precision="f32")
    buf = g.new_gradient_buffer()
    for r in range(w.rounds):
        for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
            counts = w.stage_counts(r, stage)
            for wk in range(w.workers):
                for mb in range(counts[wk]):
                    sp = w.grad_spec(r, stage, wk, mb)
                    synth.device_grad_bf16(buf, sp, 0)
                    g.add_microbatch(wk, buf)
                    o.add_microbatch(wk, synth.host_grad_bf16(sp, 0, w.n))
            if stage == synth.STAGE_TILDE:
                if scheme == "acco":
                    g.finish_half()
                    o.finish_half()
            else:
                g.finish_round()
                o.finish_round()
        torch.cuda.synchronize()
        for name in ("theta", "m", "v"):
            assert bit_mismatches(getattr(g, name).cpu().numpy(), getattr(o, name)) == 0, name
        assert bit_mismatches(g.params_f32.cpu().numpy(), o.params) == 0
        assert np.array_equal(bits_of(g.params_bf16), o.params_bf16)
