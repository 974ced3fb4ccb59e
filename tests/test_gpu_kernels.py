"""Element-by-element parity of each C-ABI entry point with the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest

import oracle
import synth
from parity import (adam_state, assert_bf16_close, assert_bf16_within_bound, assert_f32_close,
                    assert_theta_within_bound, bf16_tensor, bit_mismatches, bits_of, theta_bound)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SIZES = [0, 1, 3, 4, 7, 8, 9, 63, 64, 65, 1000, 4096 + 5, (1 << 20), (1 << 20) + 37]
DEFAULT_SHAPE = (64, 1, 0)       # the library's default: one wavefront per workgroup, no loop
SHAPES = [DEFAULT_SHAPE, (256, 1, 0), (256, 2, 0), (512, 4, 0), (256, 4, 2), (128, 2, 1)]


@pytest.fixture(scope="module")
def acco():
    import paper_2406_02613_amd as A
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    A.binding.lib()          # fails loudly if libacco.so is missing
    return A


@pytest.fixture(autouse=True)
def _default_launch_settings(acco):
    """Tests change the process-wide launch settings; whatever a test did (or however it
    ended), the next one starts from the library's defaults."""
    yield
    acco.reset_launch_settings()


def dev(a: np.ndarray):
    return torch.from_numpy(a.copy()).cuda()


def log(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ generator


def test_device_generator_matches_host_generator_bit_for_bit():
    for name in ("tiny", "gpt2s", "1b", "7b_hetero"):
        w = synth.WORKLOADS[name]
        for j0, n in ((0, 70_001), (w.n - 50_003, 50_003)):
            log("generator", name, j0, n)
            sp = w.grad_spec(2, 1, w.workers - 1, 1)
            g = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            synth.device_grad_bf16(g, sp, j0)
            assert np.array_equal(bits_of(g), synth.host_grad_bf16(sp, j0, n))
            t = torch.empty(n, dtype=torch.float32, device="cuda")
            w.device_theta(t, j0)
            assert np.array_equal(t.cpu().numpy().view(np.uint32), w.host_theta(j0, n).view(np.uint32))
    sp = synth.WORKLOADS["1b"].warm_spec(77)
    g = torch.empty(4099, dtype=torch.bfloat16, device="cuda")
    synth.device_grad_bf16(g, sp, 123_456_789)
    assert np.array_equal(bits_of(g), synth.host_grad_bf16(sp, 123_456_789, 4099))


# ------------------------------------------------------------------ accumulate / cast / reduce


def _rand_bf16(rng, n, scale=1e-3):
    x = (rng.standard_normal(n) * scale).astype(np.float32)
    return oracle.cast(x)


@pytest.mark.parametrize("shape", SHAPES)
def test_accumulate_is_bit_exact(acco, shape):
    acco.set_launch_shape("accumulate", *shape)
    rng = np.random.default_rng(1)
    for n in SIZES:
        log("accumulate", shape, n)
        acc_h = np.full(n, 7.0, np.float32)
        acc_d = dev(acc_h)
        cnt = acco.Counter(0)
        for k in range(3):
            g = _rand_bf16(rng, n)
            if n:
                g[0] = 0x8000                      # -0 must survive an init
            oracle.accumulate(acc_h, g, init=(k == 0))
            acco.acco_accumulate(acc_d, bf16_tensor(g), k == 0, cnt)
            assert cnt.value == k + 1
        assert bit_mismatches(acc_d.cpu().numpy(), acc_h) == 0


def test_cast_all_fp32_classes_bit_exact(acco):
    # every bf16 pattern combined with low halves below / at / above the rounding tie, which
    # covers zeros, denormals, infinities, NaNs and the overflow to infinity
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    src = (hi[:, None] | lows[None, :]).ravel().view(np.float32)
    want = oracle.cast(src)
    out = torch.empty(src.size, dtype=torch.bfloat16, device="cuda")
    acco.acco_cast_params(out, dev(src))
    got = bits_of(out)
    nan = np.isnan(src)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0)
    assert np.array_equal(got[nan], want[nan])       # same quieting as the oracle


@pytest.mark.parametrize("shape", SHAPES)
def test_cast_sizes(acco, shape):
    acco.set_launch_shape("cast", *shape)
    rng = np.random.default_rng(2)
    for n in SIZES:
        log("cast", shape, n)
        x = (rng.standard_normal(n) * np.exp(rng.uniform(-30, 30, n))).astype(np.float32)
        out = torch.full((n,), 1.0, dtype=torch.bfloat16, device="cuda")
        acco.acco_cast_params(out, dev(x))
        assert np.array_equal(bits_of(out), oracle.cast(x))


@pytest.mark.parametrize("shape", SHAPES[:4])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("W", [1, 2, 8, 9, 16, 17, 32, 33, 64])
def test_reduce_is_bit_exact_in_worker_order(acco, shape, dtype, W):
    acco.set_launch_shape("reduce", *shape)
    rng = np.random.default_rng(3 + W)
    for n in (0, 1, 5, 64, 1000, 4096 + 7, 300_003):
        log("reduce", shape, dtype, W, n)
        if dtype == "bf16":
            sh_h = [_rand_bf16(rng, n, 1.0) for _ in range(W)]
            sh_d = [bf16_tensor(s) for s in sh_h]
        else:
            sh_h = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
            sh_d = [dev(s) for s in sh_h]
        if n:
            # order-sensitive lanes: 2^24 + 1 + 1 ... only the left-to-right sum gives 2^24
            big = np.float32(2.0 ** 24)
            for k in range(W):
                val = big if k == 0 else np.float32(1.0)
                if dtype == "bf16":
                    sh_h[k][0] = oracle.cast(np.array([val], np.float32))[0]
                else:
                    sh_h[k][0] = val
            sh_d = [bf16_tensor(s) if dtype == "bf16" else dev(s) for s in sh_h]
        g_h = np.full(n, 3.0, np.float32)
        g_d = dev(g_h)
        tot = acco.Counter(99)
        counts = list(range(1, W + 1))
        oracle.reduce(g_h, sh_h, accumulate_=False)
        acco.acco_reduce_shards(g_d, sh_d, False, counts, tot)
        assert tot.value == sum(counts)
        assert bit_mismatches(g_d.cpu().numpy(), g_h) == 0
        oracle.reduce(g_h, sh_h[::-1], accumulate_=True)
        acco.acco_reduce_shards(g_d, sh_d[::-1], True, counts, tot)
        assert tot.value == 2 * sum(counts)
        assert bit_mismatches(g_d.cpu().numpy(), g_h) == 0


# ------------------------------------------------------------------ estimate / commit


def _state(rng, n, kind):
    return adam_state(rng, n, kind)


HYPERS = [dict(lr=6e-4, b1=0.9, b2=0.95, eps=1e-8, wd=0.1),
          dict(lr=2e-5, b1=0.9, b2=0.95, eps=1e-8, wd=0.0),
          dict(lr=0.0, b1=0.9, b2=0.999, eps=1e-6, wd=0.3),
          dict(lr=1e-2, b1=0.0, b2=0.5, eps=1e-3, wd=0.01)]


@pytest.mark.parametrize("shape", SHAPES)
def test_commit_matches_both_oracle_forms(acco, shape):
    acco.set_launch_shape("commit", *shape)
    rng = np.random.default_rng(4)
    exact = True
    for n in SIZES:
        for hi, h in enumerate(HYPERS):
            for kind, step, count in (("cold", 0, 1), ("warm", 6, 32), ("warm", 1000, 37)):
                if n > 100_000 and (hi > 1 or step == 6):
                    continue
                log("commit", shape, n, hi, kind, step, count)
                theta, m, v, gsum = _state(rng, n, kind)
                ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
                ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
                td, md, vd, gd = dev(theta), dev(m), dev(v), dev(gsum)
                out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
                st = acco.Counter(step)
                acco.acco_commit_step(td, md, vd, gd, ghp, st, count, theta_bf16=out)
                assert st.value == step + 1
                assert bit_mismatches(gd.cpu().numpy(), gsum) == 0       # input untouched
                got = [x.cpu().numpy() for x in (td, md, vd)]
                got_b = bits_of(out)
                # the bf16 copy is the RNE rounding of the fp32 theta the kernel itself wrote
                assert np.array_equal(got_b, oracle.cast(got[0]))
                for prec in ("f64", "f32"):
                    t2, m2, v2 = theta.copy(), m.copy(), v.copy()
                    want_b = oracle.commit(t2, m2, v2, gsum, ohp, step + 1, count, precision=prec)
                    assert_f32_close(got[0], t2, f"theta vs {prec}")
                    assert_f32_close(got[1], m2, f"m vs {prec}")
                    assert_f32_close(got[2], v2, f"v vs {prec}", abs_=1e-30)
                    assert_bf16_close(got_b, want_b, f"bf16 theta vs {prec}")
                    if prec == "f32":
                        exact &= (bit_mismatches(got[0], t2) + bit_mismatches(got[1], m2)
                                  + bit_mismatches(got[2], v2)) == 0
                        exact &= np.array_equal(got_b, want_b)
                # without the fused output the fp32 results are the same bits
                td2, md2, vd2 = dev(theta), dev(m), dev(v)
                acco.acco_commit_step(td2, md2, vd2, gd, ghp, acco.Counter(step), count)
                assert bit_mismatches(td2.cpu().numpy(), got[0]) == 0
                assert bit_mismatches(md2.cpu().numpy(), got[1]) == 0
                assert bit_mismatches(vd2.cpu().numpy(), got[2]) == 0
    log("commit bit-exact with the binary32 oracle form:", exact)
    # same operations, same order, each correctly rounded: the binary32 form is reproduced
    assert exact


@pytest.mark.parametrize("shape", SHAPES)
def test_estimate_reads_only_and_matches_oracle(acco, shape):
    acco.set_launch_shape("estimate", *shape)
    rng = np.random.default_rng(5)
    for n in SIZES:
        for h in HYPERS[:2]:
            log("estimate", shape, n, h["lr"])
            theta, m, v, gsum = _state(rng, n, "warm")
            ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
            ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
            td, md, vd, gd = dev(theta), dev(m), dev(v), dev(gsum)
            o32 = torch.empty(n, dtype=torch.float32, device="cuda")
            o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            acco.acco_estimate_step(td, md, vd, gd, ghp, 41, 12, theta_tilde_f32=o32,
                                    theta_tilde_bf16=o16)
            for d, h_ in ((td, theta), (md, m), (vd, v), (gd, gsum)):
                assert bit_mismatches(d.cpu().numpy(), h_) == 0
            for prec in ("f64", "f32"):
                w32, w16 = oracle.estimate(theta, m, v, gsum, ohp, 42, 12, precision=prec)
                assert_f32_close(o32.cpu().numpy(), w32, f"theta~ vs {prec}")
                assert_bf16_close(bits_of(o16), w16, f"bf16 theta~ vs {prec}")
            assert bit_mismatches(o32.cpu().numpy(), w32) == 0
            assert np.array_equal(bits_of(o16), w16)
            # single outputs give the same values
            a32 = torch.empty_like(o32)
            a16 = torch.empty_like(o16)
            acco.acco_estimate_step(td, md, vd, gd, ghp, 41, 12, theta_tilde_f32=a32)
            acco.acco_estimate_step(td, md, vd, gd, ghp, 41, 12, theta_tilde_bf16=a16)
            assert torch.equal(a32.view(torch.int32), o32.view(torch.int32))
            assert torch.equal(a16.view(torch.int16), o16.view(torch.int16))
            # and the estimate is what a commit from the same state would write
            c16 = torch.empty_like(o16)
            acco.acco_commit_step(td, md, vd, gd, ghp, acco.Counter(41), 12, theta_bf16=c16)
            assert torch.equal(td.view(torch.int32), o32.view(torch.int32))
            assert torch.equal(c16.view(torch.int16), o16.view(torch.int16))


WIDE_CASES = [(0, 0, 1), (0, 6, 32), (0, 1000, 37), (1, 0, 1), (1, 41, 12), (3, 6, 32)]


def _same_bits_nan_aware(got: np.ndarray, want: np.ndarray) -> bool:
    """fp32 arrays: NaNs in the same places (payloads may differ), every other lane bit-equal."""
    nan = np.isnan(want)
    return bool(np.array_equal(np.isnan(got), nan)
                and np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan]))


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (256, 2, 0), (512, 4, 0)])
def test_step_kernels_on_unrestricted_optimizer_states(acco, shape):
    """States that no run of Adam need have produced: m and v independent of each other,
    |m| / sqrt(v) up to 1e3, zero and denormal v under a non-zero m, and theta chosen to cancel
    against the step.  All four step entry points must reproduce the binary32 form bit for bit;
    against the binary64 form theta' is held to the bound derived from the arithmetic
    (16 * 2^-24 * (|theta| + |Adam step|), the step's numerator taken term by term), since the
    plain relative tolerance cannot hold where theta' is the residue of a cancellation; m and v
    keep the plain tolerance."""
    for e in ("estimate", "commit", "reduce_estimate", "reduce_commit"):
        acco.set_launch_shape(e, *shape)
    rng = np.random.default_rng(21)
    W = 3
    outside_plain = 0

    def check(got_theta, got_m, got_v, got_b16, state, gsum, h, ohp, index, count, committed):
        """One update from `state` on `gsum`: GPU results against both oracle forms."""
        nonlocal outside_plain
        theta, m, v = state
        bound = theta_bound(theta, m, v, gsum, h, index, count)
        t32, m32, v32 = theta.copy(), m.copy(), v.copy()
        b32 = oracle.commit(t32, m32, v32, gsum, ohp, index, count, precision="f32")
        t64, m64, v64 = theta.copy(), m.copy(), v.copy()
        b64 = oracle.commit(t64, m64, v64, gsum, ohp, index, count, precision="f64")
        assert _same_bits_nan_aware(got_theta, t32), "theta vs binary32 form"
        nan = np.isnan(t32)
        assert np.array_equal(got_b16[~nan], b32[~nan]), "bf16 vs binary32 form"
        assert np.array_equal(got_b16, oracle.cast(got_theta))
        assert_theta_within_bound(got_theta, t64, bound, "theta vs f64")
        assert_bf16_within_bound(got_b16, b64, t64, bound, "bf16 vs f64")
        if committed:
            assert _same_bits_nan_aware(got_m, m32) and _same_bits_nan_aware(got_v, v32)
            assert_f32_close(got_m, m64, "m vs f64")
            assert_f32_close(got_v, v64, "v vs f64", abs_=1e-30)
        else:                                            # a speculative step commits nothing
            assert bit_mismatches(got_m, m) == 0 and bit_mismatches(got_v, v) == 0
        err = np.abs(got_theta.astype(np.float64) - t64)
        with np.errstate(invalid="ignore"):
            plain = (err <= 1e-9) | (err <= 2e-6 * np.abs(t64)) | np.isnan(t64)
        outside_plain += int(np.count_nonzero(~plain))

    for n in (1, 17, 1000, 4096 + 5, (1 << 18) + 37):
        for hi, step, count in WIDE_CASES:
            h = HYPERS[hi]
            log("wide states", shape, n, hi, step, count)
            ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
            ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
            # --- acco_estimate_step and acco_commit_step on a given gradient sum
            theta, m, v, gsum = adam_state(rng, n, "wide", h, step + 1, count)
            td, md, vd, gd = dev(theta), dev(m), dev(v), dev(gsum)
            o32 = torch.empty(n, dtype=torch.float32, device="cuda")
            o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            acco.acco_estimate_step(td, md, vd, gd, ghp, step, count, theta_tilde_f32=o32,
                                    theta_tilde_bf16=o16)
            check(o32.cpu().numpy(), md.cpu().numpy(), vd.cpu().numpy(), bits_of(o16),
                  (theta, m, v), gsum, h, ohp, step + 1, count, committed=False)
            assert bit_mismatches(td.cpu().numpy(), theta) == 0
            st = acco.Counter(step)
            acco.acco_commit_step(td, md, vd, gd, ghp, st, count, theta_bf16=o16)
            assert st.value == step + 1
            check(td.cpu().numpy(), md.cpu().numpy(), vd.cpu().numpy(), bits_of(o16),
                  (theta, m, v), gsum, h, ohp, step + 1, count, committed=True)
            # --- the fused forms: the gradient sums come from W bf16 shards per stage
            s1 = [_rand_bf16(rng, n, 2e-4) for _ in range(W)]
            s2 = [_rand_bf16(rng, n, 2e-4) for _ in range(W)]
            d1, d2 = [bf16_tensor(x) for x in s1], [bf16_tensor(x) for x in s2]
            c1, c2 = [count] + [0] * (W - 1), [1] * W
            g1 = np.empty(n, np.float32)
            oracle.reduce(g1, s1, accumulate_=False)
            g2 = g1.copy()
            oracle.reduce(g2, s2, accumulate_=True)
            # stage 1 on a state whose theta cancels against the step on g1 / count
            theta, m, v, _ = adam_state(rng, n, "wide", h, step + 1, count, gsum=g1)
            td, md, vd = dev(theta), dev(m), dev(v)
            gd = torch.empty(n, dtype=torch.float32, device="cuda")
            tot = acco.Counter(0)
            acco.acco_reduce_estimate_step(td, md, vd, gd, d1, c1, tot, ghp, step,
                                           theta_tilde_f32=o32, theta_tilde_bf16=o16)
            assert tot.value == count and bit_mismatches(gd.cpu().numpy(), g1) == 0
            check(o32.cpu().numpy(), md.cpu().numpy(), vd.cpu().numpy(), bits_of(o16),
                  (theta, m, v), g1, h, ohp, step + 1, count, committed=False)
            assert bit_mismatches(td.cpu().numpy(), theta) == 0
            # stage 2 on a state whose theta cancels against the step on g2 / (count + W)
            theta, m, v, _ = adam_state(rng, n, "wide", h, step + 1, count + W, gsum=g2)
            td, md, vd = dev(theta), dev(m), dev(v)
            st = acco.Counter(step)
            acco.acco_reduce_commit_step(td, md, vd, gd, d2, c2, tot, ghp, st, theta_bf16=o16)
            assert tot.value == count + W and st.value == step + 1
            check(td.cpu().numpy(), md.cpu().numpy(), vd.cpu().numpy(), bits_of(o16),
                  (theta, m, v), g2, h, ohp, step + 1, count + W, committed=True)
    # the reason for the derived bound: on these states the plain tolerance does not hold
    log("elements outside the plain 2e-6 / 1e-9 tolerance (binary32 vs binary64):", outside_plain)
    assert outside_plain > 0


def test_non_finite_inputs_propagate_like_the_oracle(acco):
    n = 64
    theta = np.linspace(-1, 1, n).astype(np.float32)
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    gsum = np.ones(n, np.float32)
    gsum[1], gsum[2], gsum[3] = np.inf, -np.inf, np.nan
    theta[4] = np.inf
    ohp = oracle.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    ghp = acco.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    td, md, vd = dev(theta), dev(m), dev(v)
    out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    acco.acco_commit_step(td, md, vd, dev(gsum), ghp, acco.Counter(0), 1, theta_bf16=out)
    want_b = oracle.commit(theta, m, v, gsum, ohp, 1, 1, precision="f32")
    for got, want in ((td, theta), (md, m), (vd, v)):
        g = got.cpu().numpy()
        assert np.array_equal(np.isnan(g), np.isnan(want))
        assert np.array_equal(g[~np.isnan(want)], want[~np.isnan(want)])
    assert_bf16_close(bits_of(out), want_b, "bf16")


def test_errors_raise_and_leave_buffers_alone(acco):
    a = torch.ones(64, dtype=torch.float32, device="cuda")
    g = torch.ones(64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(acco.AccoError):
        acco.acco_accumulate(a[1:33], g[:32], False)            # misaligned view
    with pytest.raises(acco.AccoError):
        acco.acco_commit_step(a, a, a, a, acco.make_hyper(1e-3, .9, .95, 1e-8, 0),
                              acco.Counter(0), 1)                 # aliased state
    with pytest.raises(ValueError):
        acco.acco_accumulate(a, g[:32], False)                  # length mismatch
    torch.cuda.synchronize()
    assert torch.all(a == 1.0)


# ------------------------------------------------------------------ fused entry points


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (128, 2, 1), (512, 4, 0)])
def test_accumulate_publish_equals_accumulate_then_cast(acco, shape):
    acco.set_launch_shape("accumulate_publish", *shape)
    rng = np.random.default_rng(11)
    for n in SIZES:
        for init in (False, True):
            for keep in (False, True):
                log("accumulate_publish", shape, n, init, keep)
                acc0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
                g = _rand_bf16(rng, n)
                acc_h = acc0.copy()
                oracle.accumulate(acc_h, g, init=init)
                want_comm = oracle.cast(acc_h)
                acc_d = dev(acc0)
                comm = torch.full((n,), 3.0, dtype=torch.bfloat16, device="cuda")
                cnt = acco.Counter(5)
                acco.acco_accumulate_publish(acc_d, bf16_tensor(g), comm, init, keep, cnt)
                assert cnt.value == (1 if init else 6)
                assert np.array_equal(bits_of(comm), want_comm)
                assert bit_mismatches(acc_d.cpu().numpy(), acc_h if keep else acc0) == 0
    # a first-and-only micro-batch needs no accumulator at all
    g = _rand_bf16(rng, 1001)
    comm = torch.empty(1001, dtype=torch.bfloat16, device="cuda")
    acco.acco_accumulate_publish(None, bf16_tensor(g), comm, True, False)
    assert np.array_equal(bits_of(comm), g)


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (128, 2, 1), (512, 4, 0)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("W", [1, 3, 8, 9, 16, 20, 32, 33, 64])
def test_fused_reduce_steps_equal_the_separate_calls_and_the_oracle(acco, shape, dtype, W):
    acco.set_launch_shape("reduce_estimate", *shape)
    acco.set_launch_shape("reduce_commit", *shape)
    rng = np.random.default_rng(12 + W)
    h = HYPERS[0]
    ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    for n in (0, 1, 5, 64, 1000, 4096 + 7, 200_003):
        log("fused reduce+step", shape, dtype, W, n)
        theta, m, v, _ = _state(rng, n, "warm")
        if dtype == "bf16":
            s1 = [_rand_bf16(rng, n, 2e-4) for _ in range(W)]
            s2 = [_rand_bf16(rng, n, 2e-4) for _ in range(W)]
            d1, d2 = [bf16_tensor(s) for s in s1], [bf16_tensor(s) for s in s2]
        else:
            s1 = [(rng.standard_normal(n) * 2e-4).astype(np.float32) for _ in range(W)]
            s2 = [(rng.standard_normal(n) * 2e-4).astype(np.float32) for _ in range(W)]
            d1, d2 = [dev(s) for s in s1], [dev(s) for s in s2]
        c1, c2 = list(range(1, W + 1)), list(range(2, W + 2))
        # oracle: stage 1 then stage 2
        g_h = np.empty(n, np.float32)
        oracle.reduce(g_h, s1, accumulate_=False)
        e32, e16 = oracle.estimate(theta, m, v, g_h, ohp, 8, sum(c1), precision="f32")
        g1_h = g_h.copy()
        oracle.reduce(g_h, s2, accumulate_=True)
        t_h, m_h, v_h = theta.copy(), m.copy(), v.copy()
        b16 = oracle.commit(t_h, m_h, v_h, g_h, ohp, 8, sum(c1) + sum(c2), precision="f32")
        # GPU fused
        td, md, vd = dev(theta), dev(m), dev(v)
        gd = torch.full((n,), 9.0, dtype=torch.float32, device="cuda")
        o32 = torch.empty(n, dtype=torch.float32, device="cuda")
        o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        tot, step = acco.Counter(123), acco.Counter(7)
        acco.acco_reduce_estimate_step(td, md, vd, gd, d1, c1, tot, ghp, step.value,
                                       theta_tilde_f32=o32, theta_tilde_bf16=o16)
        assert tot.value == sum(c1) and step.value == 7
        assert bit_mismatches(gd.cpu().numpy(), g1_h) == 0          # the retained stage-1 sum
        assert bit_mismatches(o32.cpu().numpy(), e32) == 0
        assert np.array_equal(bits_of(o16), e16)
        for d, h_ in ((td, theta), (md, m), (vd, v)):
            assert bit_mismatches(d.cpu().numpy(), h_) == 0         # estimate commits nothing
        only16 = torch.empty_like(o16)
        acco.acco_reduce_estimate_step(td, md, vd, gd, d1, c1, acco.Counter(0), ghp, 7,
                                       theta_tilde_bf16=only16)
        assert torch.equal(only16.view(torch.int16), o16.view(torch.int16))
        c16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        acco.acco_reduce_commit_step(td, md, vd, gd, d2, c2, tot, ghp, step, theta_bf16=c16)
        assert tot.value == sum(c1) + sum(c2) and step.value == 8
        assert bit_mismatches(td.cpu().numpy(), t_h) == 0
        assert bit_mismatches(md.cpu().numpy(), m_h) == 0
        assert bit_mismatches(vd.cpu().numpy(), v_h) == 0
        assert np.array_equal(bits_of(c16), b16)
        if W <= 8:
            assert bit_mismatches(gd.cpu().numpy(), g1_h) == 0      # gsum only read
        # against the binary64 form too
        t64, m64, v64 = theta.copy(), m.copy(), v.copy()
        oracle.commit(t64, m64, v64, g_h, ohp, 8, sum(c1) + sum(c2), precision="f64")
        assert_f32_close(td.cpu().numpy(), t64, "theta vs f64")
        assert_f32_close(md.cpu().numpy(), m64, "m vs f64")
        assert_f32_close(vd.cpu().numpy(), v64, "v vs f64", abs_=1e-30)


def test_buffers_that_start_inside_an_allocation_and_guard_bands(acco):
    """Every array is a view that starts 16 bytes (or a few multiples) into a larger allocation;
    the elements just before and just after each view must come out untouched."""
    rng = np.random.default_rng(88)
    W, n, pad = 3, 70_001, 64                       # ragged: 70,001 = 4 * 17,500 + 1
    ohp = oracle.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    ghp = acco.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)

    def view(host, lead):                            # lead elements of guard before the data
        dt = torch.bfloat16 if host.dtype == np.uint16 else torch.float32
        big = torch.full((lead + n + pad,), 3.0, dtype=dt, device="cuda")
        v = big[lead:lead + n]
        v.copy_(bf16_tensor(host) if host.dtype == np.uint16 else dev(host))
        return big, v

    def guards_intact(big, lead):
        return bool(torch.all(big[:lead] == 3.0)) and bool(torch.all(big[lead + n:] == 3.0))

    theta, m, v, _ = _state(rng, n, "warm")
    grads = [[_rand_bf16(rng, n) for _ in range(2)] for _ in range(W)]
    # oracle
    acc_h = [np.empty(n, np.float32) for _ in range(W)]
    for w in range(W):
        oracle.accumulate(acc_h[w], grads[w][0], init=True)
        oracle.accumulate(acc_h[w], grads[w][1], init=False)
    comm_h = [oracle.cast(a) for a in acc_h]
    gz = np.zeros(n, np.float32)                     # stage-2 form: shards added onto gsum = 0
    oracle.reduce(gz, comm_h, accumulate_=True)
    t_h, m_h, v_h = theta.copy(), m.copy(), v.copy()
    # GPU: fp32 views lead by 4, 8, 12, ... elements, bf16 views by 8, 16, ...
    bt, td = view(theta, 4)
    bm, md = view(m, 8)
    bv, vd = view(v, 12)
    bg, gd = view(np.zeros(n, np.float32), 16)
    bo, od = view(np.zeros(n, np.uint16), 24)
    comm, bigs = [], [(bt, 4), (bm, 8), (bv, 12), (bg, 16), (bo, 24)]
    for w in range(W):
        ba, ad = view(np.zeros(n, np.float32), 4 * (w + 1))
        bc, cd = view(np.zeros(n, np.uint16), 8 * (w + 1))
        b0, g0 = view(grads[w][0], 8 * (w + 2))
        b1, g1 = view(grads[w][1], 8 * (w + 3))
        bigs += [(ba, 4 * (w + 1)), (bc, 8 * (w + 1)), (b0, 8 * (w + 2)), (b1, 8 * (w + 3))]
        cnt = acco.Counter(0)
        acco.acco_accumulate(ad, g0, True, cnt)
        acco.acco_accumulate_publish(ad, g1, cd, False, True, cnt)
        assert bit_mismatches(ad.cpu().numpy(), acc_h[w]) == 0
        comm.append(cd)
    b16 = oracle.commit(t_h, m_h, v_h, gz, ohp, 3, 2 * W, precision="f32")
    step, tot = acco.Counter(2), acco.Counter(0)
    acco.acco_reduce_commit_step(td, md, vd, gd, comm, [2] * W, tot, ghp, step, theta_bf16=od)
    assert step.value == 3 and tot.value == 2 * W
    for d, h_ in ((td, t_h), (md, m_h), (vd, v_h)):
        assert bit_mismatches(d.cpu().numpy(), h_) == 0
    assert np.array_equal(bits_of(od), b16)
    for big, lead in bigs:
        assert guards_intact(big, lead)
    # a view that starts 4 bytes in is refused, not mis-launched
    with pytest.raises(acco.AccoError):
        acco.acco_cast_params(od, bt[1:1 + n])


# ------------------------------------------------------------------ blocked state layout


@pytest.mark.parametrize("block", [4, 64, 4096])
@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (128, 2, 1), (512, 4, 0)])
def test_blocked_state_gives_the_same_bits_as_planar(acco, block, shape):
    for e in ("reduce", "estimate", "commit", "reduce_estimate", "reduce_commit"):
        acco.set_launch_shape(e, *shape)
    rng = np.random.default_rng(30 + block)
    h = HYPERS[0]
    ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    W = 3
    for n in (1, 3, 5, block - 1, block, block + 1, 3 * block + 7, 100_003, (1 << 18) + 37):
        if n < 1:
            continue
        log("blocked", block, shape, n)
        theta, m, v, _ = _state(rng, n, "warm")
        s1 = [_rand_bf16(rng, n, 2e-4) for _ in range(W)]
        s2 = [_rand_bf16(rng, n, 2e-4) for _ in range(W)]
        d1, d2 = [bf16_tensor(s) for s in s1], [bf16_tensor(s) for s in s2]
        c1, c2 = [1, 2, 3], [2, 2, 2]
        # oracle, planar by definition
        g_h = np.empty(n, np.float32)
        oracle.reduce(g_h, s1, accumulate_=False)
        e32, e16 = oracle.estimate(theta, m, v, g_h, ohp, 4, sum(c1), precision="f32")
        oracle.reduce(g_h, s2, accumulate_=True)
        t_h, m_h, v_h = theta.copy(), m.copy(), v.copy()
        b16 = oracle.commit(t_h, m_h, v_h, g_h, ohp, 4, sum(c1) + sum(c2), precision="f32")
        for fused in (False, True):
            st = acco.BlockedState(n, block)
            st.buf.fill_(123.0)                    # padding and gaps must never be touched
            for name, arr in (("theta", theta), ("m", m), ("v", v)):
                st.load(name, dev(arr))
            guard = st.buf.clone()
            o32 = torch.empty(n, dtype=torch.float32, device="cuda")
            o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            c16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            tot, step = acco.Counter(0), acco.Counter(3)
            if fused:
                acco.acco_reduce_estimate_step(st.theta, st.m, st.v, st.gsum, d1, c1, tot, ghp, 3,
                                               theta_tilde_f32=o32, theta_tilde_bf16=o16, n=n)
                acco.acco_reduce_commit_step(st.theta, st.m, st.v, st.gsum, d2, c2, tot, ghp, step,
                                             theta_bf16=c16, n=n)
            else:
                acco.acco_reduce_shards(st.gsum, d1, False, c1, tot, n=n)
                acco.acco_estimate_step(st.theta, st.m, st.v, st.gsum, ghp, 3, tot.value,
                                        theta_tilde_f32=o32, theta_tilde_bf16=o16, n=n)
                acco.acco_reduce_shards(st.gsum, d2, True, c2, tot, n=n)
                acco.acco_commit_step(st.theta, st.m, st.v, st.gsum, ghp, step, tot.value,
                                      theta_bf16=c16, n=n)
            assert tot.value == 12 and step.value == 4
            assert bit_mismatches(o32.cpu().numpy(), e32) == 0
            assert np.array_equal(bits_of(o16), e16)
            assert np.array_equal(bits_of(c16), b16)
            assert bit_mismatches(st.planar("theta").cpu().numpy(), t_h) == 0
            assert bit_mismatches(st.planar("m").cpu().numpy(), m_h) == 0
            assert bit_mismatches(st.planar("v").cpu().numpy(), v_h) == 0
            if not fused:
                assert bit_mismatches(st.planar("gsum").cpu().numpy(), g_h) == 0
            # nothing outside the n logical elements of each component was written
            flat_new = st.buf.reshape(st.blocks, 4, block)
            flat_old = guard.reshape(st.blocks, 4, block)
            rem = n - (st.blocks - 1) * block
            if rem < block:
                assert torch.equal(flat_new[-1, :, rem:], flat_old[-1, :, rem:])


def test_maximum_worker_count(acco):
    # 64 shards: eight launches of eight for the plain reduction, seven plus the fused one for
    # the fused steps; order stays ascending throughout
    rng = np.random.default_rng(64)
    n, W = 10_007, 64
    sh = [_rand_bf16(rng, n, 1.0) for _ in range(W)]
    sh[0][0] = oracle.cast(np.array([2.0 ** 24], np.float32))[0]
    for k in range(1, W):
        sh[k][0] = oracle.cast(np.array([1.0], np.float32))[0]
    dsh = [bf16_tensor(s) for s in sh]
    counts = [1] * W
    g_h = np.empty(n, np.float32)
    oracle.reduce(g_h, sh, accumulate_=False)
    assert g_h[0] == np.float32(2.0 ** 24)
    g_d = torch.empty(n, dtype=torch.float32, device="cuda")
    tot = acco.Counter(0)
    acco.acco_reduce_shards(g_d, dsh, False, counts, tot)
    assert tot.value == 64 and bit_mismatches(g_d.cpu().numpy(), g_h) == 0
    theta, m, v, _ = _state(rng, n, "warm")
    h = HYPERS[0]
    ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    td, md, vd = dev(theta), dev(m), dev(v)
    o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    g2 = torch.empty(n, dtype=torch.float32, device="cuda")
    acco.acco_reduce_estimate_step(td, md, vd, g2, dsh, counts, tot, ghp, 0, theta_tilde_bf16=o16)
    assert bit_mismatches(g2.cpu().numpy(), g_h) == 0
    _, w16 = oracle.estimate(theta, m, v, g_h, ohp, 1, 64, want_f32=False, precision="f32")
    assert np.array_equal(bits_of(o16), w16)
    step = acco.Counter(0)
    acco.acco_reduce_commit_step(td, md, vd, g2, dsh, counts, tot, ghp, step, theta_bf16=o16)
    oracle.reduce(g_h, sh, accumulate_=True)
    b16 = oracle.commit(theta, m, v, g_h, ohp, 1, 128, precision="f32")
    assert tot.value == 128 and step.value == 1
    assert bit_mismatches(td.cpu().numpy(), theta) == 0 and np.array_equal(bits_of(o16), b16)
    with pytest.raises(acco.AccoError):
        acco.acco_reduce_shards(g_d, dsh + [dsh[0]], False)          # 65 workers


def test_indexing_beyond_two_to_the_31_elements(acco):
    # element indices above 2^31 and byte offsets above 2^33: the cast and the committed step
    # (blocked state) on a 2^31 + 37 element shard, checked on sampled ranges
    n = (1 << 31) + 37
    w = synth.Workload(name="huge", n=n, workers=1, rounds=1, grad_std=1e-3, seed=31)
    slices = [(0, 4099), ((1 << 31) - 2051, (1 << 31) + 37), ((1 << 30) + 3, (1 << 30) + 4100)]
    log("huge shard", n)
    src = torch.empty(n, dtype=torch.float32, device="cuda")
    w.device_theta(src)
    out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    acco.acco_cast_params(out, src)
    for a, b in slices:
        assert np.array_equal(bits_of(out[a:b]), oracle.cast(w.host_theta(a, b - a))), (a, b)
    del out
    # committed step from m = v = 0 with gsum = the same stream scaled (any values will do)
    st = acco.BlockedState(n)
    st.load("theta", src)
    st.load("gsum", src)
    del src
    h = HYPERS[0]
    ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    acco.acco_commit_step(st.theta, st.m, st.v, st.gsum, ghp, acco.Counter(0), 16, theta_bf16=o16,
                          n=n)
    theta_p, m_p, v_p = st.planar("theta"), st.planar("m"), st.planar("v")
    for a, b in slices:
        t = w.host_theta(a, b - a)
        g = t.copy()
        m = np.zeros(b - a, np.float32)
        v = np.zeros(b - a, np.float32)
        b16 = oracle.commit(t, m, v, g, ohp, 1, 16, precision="f32")
        assert bit_mismatches(theta_p[a:b].cpu().numpy(), t) == 0, (a, b)
        assert bit_mismatches(m_p[a:b].cpu().numpy(), m) == 0
        assert bit_mismatches(v_p[a:b].cpu().numpy(), v) == 0
        assert np.array_equal(bits_of(o16[a:b]), b16)


def test_random_hyper_parameters_steps_and_counts_stay_bit_exact(acco):
    # a randomised sweep over the scalars the host folds (bias corrections at large step
    # indices, odd counts, extreme betas): the kernel must keep reproducing the binary32 form
    rng = np.random.default_rng(77)
    n = 8192 + 5
    for trial in range(60):
        lr = float(10 ** rng.uniform(-6, -1))
        b1 = float(rng.choice([0.0, 0.5, 0.9, 0.99, 0.999]))
        b2 = float(rng.choice([0.0, 0.9, 0.95, 0.999, 0.9999]))
        eps = float(10 ** rng.uniform(-12, -3))
        wd = float(rng.choice([0.0, 0.01, 0.1, 1.0]))
        step = int(rng.choice([0, 1, 2, 9, 99, 999, 12_345, 999_999, 10 ** 9]))
        count = int(rng.choice([1, 2, 3, 5, 7, 32, 37, 1000, 2 ** 20 + 1, 2 ** 40]))
        theta, m, v, gsum = _state(rng, n, "warm")
        gsum = (gsum * np.float32(min(count, 1000))).astype(np.float32)
        ohp = oracle.make_hyper(lr, b1, b2, eps, wd)
        ghp = acco.make_hyper(lr, b1, b2, eps, wd)
        td, md, vd, gd = dev(theta), dev(m), dev(v), dev(gsum)
        o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        acco.acco_estimate_step(td, md, vd, gd, ghp, step, count, theta_tilde_bf16=o16)
        _, w16 = oracle.estimate(theta, m, v, gsum, ohp, step + 1, count, want_f32=False,
                                 precision="f32")
        assert np.array_equal(bits_of(o16), w16), (trial, lr, b1, b2, eps, wd, step, count)
        acco.acco_commit_step(td, md, vd, gd, ghp, acco.Counter(step), count)
        oracle.commit(theta, m, v, gsum, ohp, step + 1, count, want_bf16=False, precision="f32")
        bad = (bit_mismatches(td.cpu().numpy(), theta) + bit_mismatches(md.cpu().numpy(), m)
               + bit_mismatches(vd.cpu().numpy(), v))
        assert bad == 0, (trial, lr, b1, b2, eps, wd, step, count)


def test_degenerate_cases_of_the_method(acco):
    n = 1003
    rng = np.random.default_rng(5)
    # eps = 0 with a zero gradient and zero moments: 0/0, NaN on both sides (payloads may differ)
    theta = rng.standard_normal(n).astype(np.float32)
    z = np.zeros(n, np.float32)
    td, md, vd, gd = dev(theta), dev(z), dev(z), dev(z)
    acco.acco_commit_step(td, md, vd, gd, acco.make_hyper(1e-3, 0.9, 0.95, 0.0, 0.0),
                          acco.Counter(0), 1)
    t2, m2, v2 = theta.copy(), z.copy(), z.copy()
    oracle.commit(t2, m2, v2, z, oracle.make_hyper(1e-3, 0.9, 0.95, 0.0, 0.0), 1, 1,
                  want_bf16=False, precision="f32")
    assert np.isnan(t2).all() and torch.isnan(td).all().item()
    assert not torch.any(md != 0).item() and not torch.any(vd != 0).item()
    # one worker, one micro-batch per stage: the round collapses to publish + step
    w = synth.Workload(name="deg", n=n, workers=1, rounds=2, grad_std=1e-3, k_fixed=2, seed=3)
    h = w.hyper
    own = acco.ShardOwner(n, 1, acco.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                          fused_publish=True, fused_reduce=True, blocked_state=True)
    th0 = w.host_theta(0, n)
    own.set_state("theta", dev(th0))
    ref = oracle.OracleShard(th0, 1, oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps,
                                                       h.weight_decay), precision="f32")
    for r in range(w.rounds):
        for stage in (1, 2):
            g = synth.host_grad_bf16(w.grad_spec(r, stage, 0, 0), 0, n)
            own.add_microbatch(0, bf16_tensor(g), last=True)
            ref.add_microbatch(0, g)
            (own.stage1 if stage == 1 else own.stage2)()
            (ref.stage1 if stage == 1 else ref.stage2)()
    assert bit_mismatches(own.get_state("theta").cpu().numpy(), ref.theta) == 0
    assert np.array_equal(bits_of(own.theta_bf16), ref.theta_bf16)
    # a worker that contributed nothing in a stage (count 0, all-zero buffer) changes no bits
    sh = [_rand_bf16(rng, n), np.zeros(n, np.uint16)]
    g1 = torch.empty(n, dtype=torch.float32, device="cuda")
    g2 = torch.empty(n, dtype=torch.float32, device="cuda")
    tot = acco.Counter(0)
    acco.acco_reduce_shards(g1, [bf16_tensor(s) for s in sh], False, [3, 0], tot)
    acco.acco_reduce_shards(g2, [bf16_tensor(sh[0])], False, [3], acco.Counter(0))
    assert tot.value == 3 and torch.equal(g1.view(torch.int32), g2.view(torch.int32))


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (256, 1, 0), (128, 2, 1), (512, 4, 0)])
def test_bf16_stash_of_the_first_micro_batch_changes_no_bits(acco, shape):
    acco.set_launch_shape("stash", *shape)
    acco.set_launch_shape("second", *shape)
    rng = np.random.default_rng(40)
    for n in SIZES + [15, 16, 17, 8 * 64 + 7]:
        log("stash", shape, n)
        g0, g1, g2 = (_rand_bf16(rng, n) for _ in range(3))
        if n > 4:
            g0[0], g1[0] = 0x8000, 0x8000          # -0 + -0 stays -0
            g0[1] = 0x7FA0                          # a signalling NaN pattern
            g0[2], g1[2] = 0x7F80, 0xFF80          # inf - inf
        d0, d1, d2 = bf16_tensor(g0), bf16_tensor(g1), bf16_tensor(g2)
        # oracle: plain fp32 accumulation, published after 1, 2 and 3 micro-batches
        acc_h = np.empty(n, np.float32)
        oracle.accumulate(acc_h, g0, init=True)
        pub1 = oracle.cast(acc_h)
        oracle.accumulate(acc_h, g1, init=False)
        acc2_h, pub2 = acc_h.copy(), oracle.cast(acc_h)
        oracle.accumulate(acc_h, g2, init=False)
        pub3 = oracle.cast(acc_h)
        cnt = acco.Counter(9)
        stash = torch.full((n,), 2.0, dtype=torch.bfloat16, device="cuda")
        comm = torch.full((n,), 2.0, dtype=torch.bfloat16, device="cuda")
        acc = torch.full((n,), 2.0, dtype=torch.float32, device="cuda")
        # one micro-batch only: published directly
        acco.acco_accumulate_first(comm, d0, True, cnt)
        assert cnt.value == 1
        got, nan = bits_of(comm), np.isnan(oracle.bf16_to_f32(pub1))
        assert np.array_equal(got[~nan], pub1[~nan]) and np.array_equal(got[nan], pub1[nan])
        # two micro-batches: stash, then second + publish
        acco.acco_accumulate_first(stash, d0, False, cnt)
        assert np.array_equal(bits_of(stash), g0)                 # a stash keeps the raw bits
        acco.acco_accumulate_second(stash, d1, comm_bf16=comm, count=cnt)
        assert cnt.value == 2
        nan2 = np.isnan(acc2_h)
        got = bits_of(comm)
        assert np.array_equal(got[~nan2], pub2[~nan2])
        assert np.all((got[nan2] & 0x7F80) == 0x7F80) and np.all((got[nan2] & 0x7F) != 0)
        # three: stash, second into the fp32 accumulator, then the ordinary fused last one
        cnt.value = 1
        acco.acco_accumulate_second(stash, d1, acc=acc, count=cnt)
        a = acc.cpu().numpy()
        assert np.array_equal(a.view(np.uint32)[~nan2], acc2_h.view(np.uint32)[~nan2])
        assert np.isnan(a[nan2]).all()
        acco.acco_accumulate_publish(acc, d2, comm, False, False, cnt)
        assert cnt.value == 3
        got = bits_of(comm)
        assert np.array_equal(got[~nan2], pub3[~nan2])


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (256, 1, 0), (128, 2, 1), (512, 4, 0)])
def test_bf16_running_sum_is_bit_exact(acco, shape):
    """The paper's buffer precision (Sec. 4): the sum is rounded to bf16 after every micro-batch."""
    acco.set_launch_shape("stash", *shape)
    acco.set_launch_shape("second", *shape)
    rng = np.random.default_rng(41)
    for n in SIZES + [15, 16, 17, 8 * 64 + 7]:
        log("bf16 running sum", shape, n)
        acc_h = np.full(n, 0x4123, np.uint16)
        acc_d = bf16_tensor(acc_h)
        cnt = acco.Counter(5)
        for k in range(4):
            g = _rand_bf16(rng, n, scale=1e-3 * (1 + 30 * (k == 2)))   # one much larger term
            if n > 4:
                g[0] = 0x8000                       # -0 survives the init and -0 + -0
                g[1] = 0x0001 if k % 2 else 0x8001  # subnormals cancel exactly
                g[2] = 0x7F00 if k < 2 else 0x0000  # overflows to +inf at the second add
            oracle.accumulate_bf16(acc_h, g, init=(k == 0))
            acco.acco_accumulate_bf16(acc_d, bf16_tensor(g), k == 0, cnt)
            assert cnt.value == k + 1
            assert np.array_equal(bits_of(acc_d), acc_h), (n, k)
        if n > 4:
            assert acc_h[0] == 0x8000 and acc_h[2] == 0x7F80
    # stagnation at 256: the closed form of a bf16 running sum of ones
    ones = torch.ones(1000, dtype=torch.bfloat16, device="cuda")
    acc = torch.empty_like(ones)
    cnt = acco.Counter(0)
    for k in range(300):
        acco.acco_accumulate_bf16(acc, ones, k == 0, cnt)
    assert cnt.value == 300 and torch.all(acc.float() == 256.0)


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (256, 2, 0), (128, 1, 3), (512, 4, 0)])
@pytest.mark.parametrize("W", [1, 3, 16, 17, 40])
def test_batched_accumulation_steps_equal_the_single_calls(acco, shape, W):
    """acco_accumulate_batch: every operation, for W workers in one call (17 and 40 need more than
    one launch), against the oracle's plain accumulation, publish and bf16 running sum."""
    Bn = acco.binding
    for e in ("accumulate", "accumulate_publish", "stash", "second", "cast"):
        acco.set_launch_shape(e, *shape)
    rng = np.random.default_rng(50 + W)
    for n in (0, 1, 7, 8, 9, 515, 4096 + 5, 100_003):
        log("batch", shape, W, n)
        g = [[_rand_bf16(rng, n) for _ in range(W)] for _ in range(3)]
        if n > 4:
            for k in range(3):
                for w in range(W):
                    g[k][w][0] = 0x8000                       # -0 + -0 stays -0
                    g[k][w][1] = 0x7FA0 if k == 0 else 0x0000  # a signalling NaN pattern
        d = [[bf16_tensor(x) for x in row] for row in g]
        # oracle: fp32 accumulators after 1, 2, 3 micro-batches and their bf16 publishes
        acc_h = [np.empty(n, np.float32) for _ in range(W)]
        pubs, accs = [], []
        for k in range(3):
            for w in range(W):
                oracle.accumulate(acc_h[w], g[k][w], init=(k == 0))
            accs.append([a.copy() for a in acc_h])
            pubs.append([oracle.cast(a) for a in acc_h])

        def same_bf16(t, want):
            got = bits_of(t)
            nan = (want & 0x7FFF) > 0x7F80
            return (np.array_equal(got[~nan], want[~nan])
                    and np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0))

        def same_f32(t, want):
            got = t.cpu().numpy()
            nan = np.isnan(want)
            return (np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])
                    and np.isnan(got[nan]).all())

        cnt = [acco.Counter(9) for _ in range(W)]
        acc = [torch.full((n,), 2.0, dtype=torch.float32, device="cuda") for _ in range(W)]
        out = [torch.full((n,), 2.0, dtype=torch.bfloat16, device="cuda") for _ in range(W)]
        stash = [torch.full((n,), 2.0, dtype=torch.bfloat16, device="cuda") for _ in range(W)]
        # fp32 path: init, add, add + publish; then a plain publish of the accumulators
        acco.acco_accumulate_batch(Bn.BATCH_ACCUMULATE_INIT, n, acc=acc, grad_bf16=d[0], counts=cnt)
        assert all(c.value == 1 for c in cnt)
        assert all(same_f32(acc[w], accs[0][w]) for w in range(W))
        acco.acco_accumulate_batch(Bn.BATCH_ACCUMULATE, n, acc=acc, grad_bf16=d[1], counts=cnt)
        assert all(same_f32(acc[w], accs[1][w]) for w in range(W))
        acco.acco_accumulate_batch(Bn.BATCH_PUBLISH, n, acc=acc, out_bf16=out, counts=cnt)
        assert all(c.value == 2 for c in cnt)
        assert all(same_bf16(out[w], pubs[1][w]) for w in range(W))
        acco.acco_accumulate_batch(Bn.BATCH_ACCUMULATE_PUBLISH, n, acc=acc, out_bf16=out,
                                   grad_bf16=d[2], counts=cnt)
        assert all(c.value == 3 for c in cnt)
        assert all(same_bf16(out[w], pubs[2][w]) for w in range(W))
        assert all(same_f32(acc[w], accs[1][w]) for w in range(W))       # accumulators only read
        # stash path: first, first + publish, second, second + publish
        acco.acco_accumulate_batch(Bn.BATCH_FIRST_PUBLISH, n, out_bf16=out, grad_bf16=d[0],
                                   counts=cnt)
        assert all(c.value == 1 for c in cnt)
        assert all(same_bf16(out[w], pubs[0][w]) for w in range(W))
        acco.acco_accumulate_batch(Bn.BATCH_FIRST, n, out_bf16=stash, grad_bf16=d[0], counts=cnt)
        assert all(np.array_equal(bits_of(stash[w]), g[0][w]) for w in range(W))   # raw bits kept
        acco.acco_accumulate_batch(Bn.BATCH_SECOND_PUBLISH, n, out_bf16=out, stash_bf16=stash,
                                   grad_bf16=d[1], counts=cnt)
        assert all(c.value == 2 for c in cnt)
        assert all(same_bf16(out[w], pubs[1][w]) for w in range(W))
        for c in cnt:
            c.value = 1
        acco.acco_accumulate_batch(Bn.BATCH_SECOND, n, acc=acc, stash_bf16=stash, grad_bf16=d[1],
                                   counts=cnt)
        assert all(same_f32(acc[w], accs[1][w]) for w in range(W))
        # bf16 running sums (the paper's buffer precision), in place
        run_h = [x.copy() for x in g[0]]
        acco.acco_accumulate_batch(Bn.BATCH_FIRST, n, out_bf16=out, grad_bf16=d[0], counts=cnt)
        for k in (1, 2):
            for w in range(W):
                oracle.accumulate_bf16(run_h[w], g[k][w], init=False)
            acco.acco_accumulate_batch(Bn.BATCH_RUNNING_BF16, n, out_bf16=out, grad_bf16=d[k],
                                       counts=cnt)
            assert all(c.value == k + 1 for c in cnt)
            assert all(same_bf16(out[w], run_h[w]) for w in range(W))
    # a buffer given twice as an output is refused, nothing is launched
    if W > 1:
        n = 64
        a = [torch.ones(n, dtype=torch.float32, device="cuda") for _ in range(W)]
        gg = [torch.ones(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)]
        with pytest.raises(acco.AccoError):
            acco.acco_accumulate_batch(Bn.BATCH_ACCUMULATE, n, acc=[a[0]] * W, grad_bf16=gg)
        torch.cuda.synchronize()
        assert torch.all(a[0] == 1.0)


@pytest.mark.parametrize("shape", [DEFAULT_SHAPE, (128, 1, 0), (256, 2, 0), (512, 4, 0)])
@pytest.mark.parametrize("block", [8, 64, 1024, 16384])
@pytest.mark.parametrize("W", [1, 3, 8, 20, 32, 40])
def test_interleaved_communication_buffers_give_the_same_bits(acco, shape, block, W):
    """The W communication buffers as the interleaved blocks of one buffer: every operation that
    publishes into them (out_layout) and every reduction that reads them (shard_layout) against
    the same calls on W separate planar buffers and against the oracle; nothing outside the
    buffers' n logical elements is written."""
    Bn = acco.binding
    for e in ("accumulate_publish", "stash", "second", "cast", "reduce", "reduce_estimate",
              "reduce_commit"):
        acco.set_launch_shape(e, *shape)
    rng = np.random.default_rng(60 + W + block)
    h = HYPERS[0]
    ohp = oracle.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    ghp = acco.make_hyper(h["lr"], h["b1"], h["b2"], h["eps"], h["wd"])
    for n in (0, 1, 7, 8, 9, block - 1, block, block + 1, 3 * block + 5, 70_001):
        if n < 0 or (block == 16384 and n > 2 * block + 100 and n != 70_001):
            continue
        log("interleaved comm", shape, block, W, n)
        g = [[_rand_bf16(rng, n, 2e-4) for _ in range(W)] for _ in range(3)]
        d = [[bf16_tensor(x) for x in row] for row in g]
        # oracle: sums after 1, 2, 3 micro-batches, their publishes, the reduced gradient
        acc_h = [np.empty(n, np.float32) for _ in range(W)]
        pubs = []
        for k in range(3):
            for w in range(W):
                oracle.accumulate(acc_h[w], g[k][w], init=(k == 0))
            pubs.append([oracle.cast(a) for a in acc_h])
        acc2 = [np.empty(n, np.float32) for _ in range(W)]
        for w in range(W):
            oracle.accumulate(acc2[w], g[0][w], init=True)
            oracle.accumulate(acc2[w], g[1][w], init=False)
        slab = acco.InterleavedShards(n, W, block)
        slab.buf.fill_(7.0)                                   # padding must never be touched
        comm = slab.shards
        stash = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)]
        acc = [dev(a) for a in acc2]

        def published(k):
            return all(np.array_equal(bits_of(slab.planar(w)), pubs[k][w]) for w in range(W))

        def padding_intact():
            rem = n - (slab.blocks - 1) * block if slab.blocks else 0
            return slab.blocks == 0 or rem == block or bool(torch.all(slab.buf[-1, :, rem:] == 7.0))

        acco.acco_accumulate_batch(Bn.BATCH_FIRST_PUBLISH, n, out_bf16=comm, grad_bf16=d[0])
        assert published(0) and padding_intact()
        acco.acco_accumulate_batch(Bn.BATCH_FIRST, n, out_bf16=stash, grad_bf16=d[0])
        acco.acco_accumulate_batch(Bn.BATCH_SECOND_PUBLISH, n, out_bf16=comm, stash_bf16=stash,
                                   grad_bf16=d[1])
        assert published(1) and padding_intact()
        acco.acco_accumulate_batch(Bn.BATCH_ACCUMULATE_PUBLISH, n, acc=acc, out_bf16=comm,
                                   grad_bf16=d[2])
        assert published(2) and padding_intact()
        acco.acco_accumulate_batch(Bn.BATCH_PUBLISH, n, acc=acc, out_bf16=comm)
        assert published(1) and padding_intact()
        # a stash may be interleaved too (FIRST keeps the raw bits)
        slab2 = acco.InterleavedShards(n, W, block)
        acco.acco_accumulate_batch(Bn.BATCH_FIRST, n, out_bf16=slab2.shards, grad_bf16=d[0])
        assert all(np.array_equal(bits_of(slab2.planar(w)), g[0][w]) for w in range(W))
        # the reductions over the interleaved buffers (comm holds the sums of two micro-batches)
        planar = [bf16_tensor(pubs[1][w]) for w in range(W)]
        counts = [2] * W
        g1 = torch.empty(n, dtype=torch.float32, device="cuda")
        g2 = torch.empty(n, dtype=torch.float32, device="cuda")
        acco.acco_reduce_shards(g1, comm, False, counts, acco.Counter(0))
        acco.acco_reduce_shards(g2, planar, False, counts, acco.Counter(0))
        g_h = np.empty(n, np.float32)
        oracle.reduce(g_h, pubs[1], accumulate_=False)
        assert bit_mismatches(g1.cpu().numpy(), g_h) == 0 and torch.equal(g1.view(torch.int32), g2.view(torch.int32))
        acco.acco_reduce_shards(g1, comm, True, counts, acco.Counter(0))
        oracle.reduce(g_h, pubs[1], accumulate_=True)
        assert bit_mismatches(g1.cpu().numpy(), g_h) == 0
        theta, m, v, _ = _state(rng, n, "warm")
        for blocked_state in (False, True):
            if blocked_state:
                st = acco.BlockedState(n, 64)
                for name, arr in (("theta", theta), ("m", m), ("v", v)):
                    st.load(name, dev(arr))
                td, md, vd, gd = st.theta, st.m, st.v, st.gsum
            else:
                td, md, vd = dev(theta), dev(m), dev(v)
                gd = torch.empty(n, dtype=torch.float32, device="cuda")
            o16 = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            tot, step = acco.Counter(0), acco.Counter(4)
            acco.acco_reduce_estimate_step(td, md, vd, gd, comm, counts, tot, ghp, step.value,
                                           theta_tilde_bf16=o16, n=n)
            g_h = np.empty(n, np.float32)
            oracle.reduce(g_h, pubs[1], accumulate_=False)
            _, e16 = oracle.estimate(theta, m, v, g_h, ohp, 5, 2 * W, want_f32=False, precision="f32")
            assert np.array_equal(bits_of(o16), e16)
            acco.acco_reduce_commit_step(td, md, vd, gd, comm, counts, tot, ghp, step,
                                         theta_bf16=o16, n=n)
            oracle.reduce(g_h, pubs[1], accumulate_=True)
            t_h, m_h, v_h = theta.copy(), m.copy(), v.copy()
            b16 = oracle.commit(t_h, m_h, v_h, g_h, ohp, 5, 4 * W, precision="f32")
            assert tot.value == 4 * W and step.value == 5
            got_t = st.planar("theta") if blocked_state else td
            assert bit_mismatches(got_t.cpu().numpy(), t_h) == 0
            assert np.array_equal(bits_of(o16), b16)
        assert padding_intact()


def test_resident_wave_bounds_change_no_bits(acco):
    """The bound on resident wavefronts (an LDS reservation) is a scheduling knob only."""
    rng = np.random.default_rng(43)
    n = (1 << 20) + 37
    hp, ohp = acco.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1), oracle.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    th = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    v = (rng.standard_normal(n) ** 2 * 1e-8).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    want = [x.copy() for x in (th, m, v)]
    want_bf16 = oracle.commit(*want, g, ohp, 7, 4, precision="f32")
    try:
        for shape, bound in (((64, 1, 0), 0), ((64, 1, 0), 3), ((64, 1, 0), 9), ((64, 1, 0), 32),
                             ((256, 1, 0), 12), ((512, 4, 2), 24), ((512, 1, 0), 9)):
            log("resident waves", shape, bound)
            acco.set_launch_shape("commit", *shape)
            acco.set_resident_waves("commit", 0)
            if bound:
                try:
                    acco.set_resident_waves("commit", bound)
                except acco.AccoError:
                    assert bound // (shape[0] // 64) < 3          # refused, not mis-launched
                    continue
            d = [dev(x) for x in (th, m, v)]
            out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            acco.acco_commit_step(*d, dev(g), hp, acco.Counter(6), 4, theta_bf16=out)
            for got, w in zip(d, want):
                assert bit_mismatches(got.cpu().numpy(), w) == 0
            assert np.array_equal(bits_of(out), want_bf16)
    finally:
        acco.reset_launch_settings()


def test_bandwidth_probes_do_what_they_say(acco):
    rng = np.random.default_rng(9)
    for n in (0, 1, 5, 4096 + 3, 100_001):
        a, b, c, d = (rng.standard_normal(n).astype(np.float32) for _ in range(4))
        da, db, dc, dd = dev(a), dev(b), dev(c), dev(d)
        out = torch.zeros(n, dtype=torch.float32, device="cuda")
        acco.binding.acco_probe_copy(out, dd)
        assert bit_mismatches(out.cpu().numpy(), d) == 0
        acco.binding.acco_probe_triad(da, db, dc, dd)
        for got, want in ((da, a + d), (db, b + d), (dc, c + d)):
            assert bit_mismatches(got.cpu().numpy(), want.astype(np.float32)) == 0
        assert bit_mismatches(dd.cpu().numpy(), d) == 0


def test_shard_longer_than_one_dispatch_of_one_wave_workgroups(acco):
    # 2^34 + 5 elements: more 64-thread tiles than one dispatch can hold work-items for, so the
    # launch falls back to the looping kernel; byte offsets go beyond 2^36
    n = (1 << 34) + 5
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < n * 6 + (8 << 30):
        pytest.skip("needs about 104 GB of free device memory")
    w = synth.Workload(name="giant", n=n, workers=1, rounds=1, seed=33)
    log("giant shard", n)
    src = torch.empty(n, dtype=torch.float32, device="cuda")
    w.device_theta(src)
    out = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    acco.acco_cast_params(out, src)
    torch.cuda.synchronize()
    for a, b in ((0, 4099), ((1 << 33) + 1, (1 << 33) + 4100), (n - 4101, n)):
        assert np.array_equal(bits_of(out[a:b]), oracle.cast(w.host_theta(a, b - a))), (a, b)
    del src, out
    torch.cuda.empty_cache()
