"""Pins for the oracle's round sequencing (Alg. 1, communication stream, one shard owner)."""
import numpy as np
import pytest
import torch

import oracle
import synth

TOL_REL, TOL_ABS = 2e-6, 1e-9


def close(a, b, rel=TOL_REL, abs_=TOL_ABS):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.all((np.abs(a - b) <= abs_) | (np.abs(a - b) <= rel * np.abs(b)))


def _hp(w: synth.Workload):
    h = w.hyper
    return oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay)


def _run_round(sh: oracle.OracleShard, w: synth.Workload, rnd: int, j0: int, n: int,
               estimate_calls: int = 1, grads=None):
    """Feed one round of w's micro-batches (slice [j0, j0+n)) through the oracle."""
    for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
        counts = w.stage_counts(rnd, stage)
        for wk in range(w.workers):
            for mb in range(counts[wk]):
                g = synth.host_grad_bf16(w.grad_spec(rnd, stage, wk, mb), j0, n)
                if grads is not None:
                    grads.append((stage, wk, g))
                sh.add_microbatch(wk, g)
        if stage == synth.STAGE_TILDE:
            if estimate_calls == 0:
                # the owner still has to take the first-half sum; only the Opt call is skipped
                oracle.reduce(sh.gsum, sh._publish(), accumulate_=False)
                sh.total = sum(sh.count)
                sh.count = [0] * sh.W
            else:
                keep = sh.count[:]
                sh.stage1()
                for _ in range(estimate_calls - 1):  # repeated speculative calls change nothing
                    oracle.estimate(sh.theta, sh.m, sh.v, sh.gsum, sh.hp, sh.step + 1, sh.total,
                                    precision=sh.precision)
                assert sum(keep) == sh.total
        else:
            sh.stage2()


TINY = synth.Workload(name="t", n=5000, workers=3, rounds=3, theta_dist="uniform",
                      theta_param=0.05, grad_std=1e-3, k_range=(2, 7), seed=11)


@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_committed_trajectory_does_not_depend_on_the_estimate(precision):
    # stage (2) starts from the same theta(t) as stage (1): running the speculative step zero,
    # one or several times leaves every committed bit the same.
    res = []
    for calls in (0, 1, 3):
        sh = oracle.OracleShard(TINY.host_theta(0, TINY.n), TINY.workers, _hp(TINY),
                                precision=precision)
        for r in range(TINY.rounds):
            _run_round(sh, TINY, r, 0, TINY.n, estimate_calls=calls)
        res.append((sh.theta.copy(), sh.m.copy(), sh.v.copy(), sh.step))
    for th, m, v, step in res[1:]:
        assert step == res[0][3] == TINY.rounds
        for a, b in zip((th, m, v), res[0][:3]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_equal_halves_make_the_estimate_equal_the_commit(precision):
    # one worker, second half identical to the first: the full sum is exactly twice the half
    # sum and the count doubles, so the normalised gradients coincide and so do the bf16 outputs.
    n = 4097
    w = synth.Workload(name="e", n=n, workers=1, rounds=1, grad_std=1e-3, k_fixed=2, seed=3)
    sh = oracle.OracleShard(w.host_theta(0, n), 1, _hp(w), precision=precision)
    g = synth.host_grad_bf16(w.grad_spec(0, 1, 0, 0), 0, n)
    sh.add_microbatch(0, g)
    sh.stage1()
    sh.add_microbatch(0, g)
    sh.stage2()
    assert np.array_equal(sh.theta_tilde_bf16, sh.theta_bf16)


def _brute_force_mean(grads, stages):
    """(sum of every listed micro-batch gradient) / (their number), in fp64, from the raw bits."""
    sel = [oracle.bf16_to_f32(g).astype(np.float64) for (st, _, g) in grads if st in stages]
    return np.sum(sel, axis=0) / len(sel), len(sel)


@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_unequal_worker_counts_normalise_by_the_total_count(precision):
    # first round from m = v = 0: m' = (1-b1) gbar, v' = (1-b2) gbar^2 with gbar the mean over
    # ALL micro-batches of all workers (fp32 communication, so no publish rounding is involved)
    sh = oracle.OracleShard(TINY.host_theta(0, TINY.n), TINY.workers, _hp(TINY),
                            precision=precision, comm_dtype="f32")
    grads = []
    _run_round(sh, TINY, 0, 0, TINY.n, grads=grads)
    gbar, cnt = _brute_force_mean(grads, (1, 2))
    assert cnt == sum(TINY.microbatches(0, k) for k in range(TINY.workers))
    assert len({TINY.microbatches(0, k) for k in range(TINY.workers)}) > 1  # really unequal
    assert close(sh.m, 0.1 * gbar, rel=1e-6, abs_=1e-11)
    assert close(sh.v, 0.05 * gbar * gbar, rel=1e-6, abs_=1e-30)


@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_estimate_uses_only_the_first_half_and_its_own_count(precision):
    sh = oracle.OracleShard(TINY.host_theta(0, TINY.n), TINY.workers, _hp(TINY),
                            precision=precision, comm_dtype="f32")
    theta0 = sh.theta.astype(np.float64)
    grads = []
    _run_round(sh, TINY, 0, 0, TINY.n, grads=grads)
    gt, cnt = _brute_force_mean(grads, (1,))
    assert cnt == sum(TINY.split(0, k)[0] for k in range(TINY.workers))
    h = TINY.hyper
    # step 1 from zero moments: closed form of the first Adam step, with decay
    want = theta0 * (1 - h.lr * h.weight_decay) - h.lr * gt / (np.abs(gt) + h.eps)
    want_bf16 = torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16)
    got = torch.from_numpy(sh.theta_tilde_bf16.view(np.int16)).view(torch.bfloat16)
    # a last-bit difference in fp32 can flip a bf16 rounding: allow one bf16 ulp, rarely
    d = np.abs(got.view(torch.int16).numpy().astype(np.int32)
               - want_bf16.view(torch.int16).numpy().astype(np.int32))
    assert d.max() <= 1 and np.mean(d != 0) < 1e-3


def test_bf16_publish_rounds_each_workers_sum_before_the_reduction():
    # brute force with torch's cast as the independent bf16 rounding
    w = synth.Workload(name="p", n=3001, workers=4, rounds=1, grad_std=1e-3, k_fixed=6, seed=5)
    sh = oracle.OracleShard(w.host_theta(0, w.n), w.workers, _hp(w), comm_dtype="bf16")
    per_worker = [np.zeros(w.n, np.float32) for _ in range(w.workers)]
    for wk in range(w.workers):
        for mb in range(3):
            g = synth.host_grad_bf16(w.grad_spec(0, 1, wk, mb), 0, w.n)
            sh.add_microbatch(wk, g)
            gf = oracle.bf16_to_f32(g)
            per_worker[wk] = gf.copy() if mb == 0 else (per_worker[wk] + gf).astype(np.float32)
    sh.stage1()
    want = np.zeros(w.n, np.float32)
    for wk in range(w.workers):
        pub = torch.from_numpy(per_worker[wk]).to(torch.bfloat16).to(torch.float32).numpy()
        want = pub.copy() if wk == 0 else (want + pub).astype(np.float32)
    assert np.array_equal(sh.gsum.view(np.uint32), want.view(np.uint32))
    assert sh.total == 12


@pytest.mark.parametrize("precision", ["f64", "f32"])
def test_rounds_follow_plain_adamw_on_the_full_batch_gradient(precision):
    # eq. (DDP) with Opt = AdamW: commit-only dynamics on the mean of all micro-batch gradients.
    w = synth.Workload(name="d", n=6000, workers=2, rounds=6, grad_std=1e-3, k_range=(2, 5),
                       seed=21)
    sh = oracle.OracleShard(w.host_theta(0, w.n), w.workers, _hp(w), precision=precision,
                            comm_dtype="f32")
    p = torch.nn.Parameter(torch.from_numpy(w.host_theta(0, w.n).copy()))
    h = w.hyper
    opt = torch.optim.AdamW([p], lr=h.lr, betas=(h.beta1, h.beta2), eps=h.eps,
                            weight_decay=h.weight_decay, foreach=False, fused=False)
    for r in range(w.rounds):
        grads = []
        _run_round(sh, w, r, 0, w.n, grads=grads)
        gbar, _ = _brute_force_mean(grads, (1, 2))
        p.grad = torch.from_numpy(gbar.astype(np.float32))
        opt.step()
    drift = w.rounds * 2.0 ** -25
    ref = p.detach().numpy()
    assert close(sh.theta, ref, rel=TOL_REL + drift, abs_=TOL_ABS + drift * 0.1)
    assert close(sh.m, opt.state[p]["exp_avg"].numpy(), rel=4e-6, abs_=1e-10)
    assert close(sh.v, opt.state[p]["exp_avg_sq"].numpy(), rel=4e-6, abs_=1e-30)
    assert sh.step == w.rounds


def test_scheduled_rounds_follow_torch_adamw_under_cosine_annealing():
    """Cosine schedule of the paper's hyper-parameter tables (App. C): the rate of update t is a
    host scalar; the oracle's rounds with it track torch's AdamW + CosineAnnealingLR."""
    T = 12                                            # short horizon: the rate really moves
    w = synth.Workload(name="s", n=4000, workers=2, rounds=T, grad_std=1e-3, k_range=(2, 4),
                       seed=23)
    h = w.hyper
    sched = lambda t: oracle.lr_cosine(h.lr, h.lr / 10, t, 0, T)      # noqa: E731
    assert abs(sched(0) - h.lr) < 1e-18 and abs(sched(T) - h.lr / 10) < 1e-18 and sched(5) > sched(6)
    sh = oracle.OracleShard(w.host_theta(0, w.n), w.workers, _hp(w), precision="f32",
                            comm_dtype="f32", lr_schedule=sched)
    p = torch.nn.Parameter(torch.from_numpy(w.host_theta(0, w.n).copy()))
    opt = torch.optim.AdamW([p], lr=h.lr, betas=(h.beta1, h.beta2), eps=h.eps,
                            weight_decay=h.weight_decay, foreach=False, fused=False)
    lrs = torch.optim.lr_scheduler.CosineAnnealingLR(opt, T_max=T, eta_min=h.lr / 10)
    for r in range(T):
        assert abs(opt.param_groups[0]["lr"] - sched(r)) <= 1e-12 * h.lr
        grads = []
        _run_round(sh, w, r, 0, w.n, grads=grads)
        gbar, _ = _brute_force_mean(grads, (1, 2))
        p.grad = torch.from_numpy(gbar.astype(np.float32))
        opt.step()
        lrs.step()
    drift = T * 2.0 ** -25
    assert close(sh.theta, p.detach().numpy(), rel=TOL_REL + drift, abs_=TOL_ABS + drift * 0.1)
    # and the schedule matters: a constant rate ends somewhere else
    const = oracle.OracleShard(w.host_theta(0, w.n), w.workers, _hp(w), precision="f32",
                               comm_dtype="f32")
    for r in range(T):
        _run_round(const, w, r, 0, w.n)
    assert not close(const.theta, sh.theta, rel=1e-4, abs_=1e-6)


def test_counters_match_a_recount_of_the_micro_batch_table():
    w = synth.WORKLOADS["7b_hetero"]
    small = synth.Workload(name="c", n=64, workers=w.workers, rounds=w.rounds, k_range=w.k_range,
                           seed=w.seed, grad_std=w.grad_std)
    sh = oracle.OracleShard(small.host_theta(0, 64), small.workers, _hp(small))
    for r in range(small.rounds):
        table = [small.microbatches(r, k) for k in range(small.workers)]
        assert all(2 <= k <= 8 for k in table)
        for stage in (1, 2):
            counts = small.stage_counts(r, stage)
            assert counts == [(k // 2 if stage == 1 else k - k // 2) for k in table]
            for wk in range(small.workers):
                for mb in range(counts[wk]):
                    sh.add_microbatch(wk, synth.host_grad_bf16(small.grad_spec(r, stage, wk, mb),
                                                               0, 64))
            assert sh.count == counts
            if stage == 1:
                sh.stage1()
                assert sh.total == sum(k // 2 for k in table) and sh.count == [0] * small.workers
            else:
                before = sh.total
                sh.stage2()
                assert before + sum(counts) == sum(table)
                assert sh.total == 0 and sh.step == r + 1


def test_slices_of_a_run_equal_the_run_on_the_whole_shard():
    # every operation is elementwise and the generator is index-addressable: running the oracle
    # on [a, b) alone gives the same bits as slicing a whole-shard run.  This is what lets the
    # full-size GPU runs be checked on sampled slices.
    w = synth.Workload(name="s", n=20_011, workers=3, rounds=2, grad_std=1e-3, k_range=(2, 4),
                       zero_frac=0.05, zero_run=64, outlier_frac=1e-2, seed=8)
    full = oracle.OracleShard(w.host_theta(0, w.n), w.workers, _hp(w), precision="f32")
    a, b = 7003, 9999
    part = oracle.OracleShard(w.host_theta(a, b - a), w.workers, _hp(w), precision="f32")
    for r in range(w.rounds):
        _run_round(full, w, r, 0, w.n)
        _run_round(part, w, r, a, b - a)
    for x, y in ((full.theta, part.theta), (full.m, part.m), (full.v, part.v)):
        assert np.array_equal(x[a:b].view(np.uint32), y.view(np.uint32))
    assert np.array_equal(full.theta_bf16[a:b], part.theta_bf16)
    assert np.array_equal(full.theta_tilde_bf16[a:b], part.theta_tilde_bf16)


def test_bf16_accumulators_equal_fp32_accumulators_for_single_microbatch_stages():
    """With one micro-batch per worker and stage, the published buffer is that gradient itself in
    either precision (bf16 -> fp32 -> bf16 is the identity), so the trajectories coincide bit for
    bit; with more micro-batches the bf16 running sum rounds after every add and only stays close."""
    one = synth.Workload(name="k2", n=3000, workers=3, rounds=2, theta_dist="uniform",
                         theta_param=0.05, grad_std=1e-3, k_range=(2, 2), seed=5)
    many = synth.Workload(name="k6", n=3000, workers=3, rounds=2, theta_dist="uniform",
                          theta_param=0.05, grad_std=1e-3, k_range=(6, 6), seed=5)
    out = {}
    for w in (one, many):
        for acc_dtype in ("f32", "bf16"):
            sh = oracle.OracleShard(w.host_theta(0, w.n), w.workers, _hp(w),
                                    precision="f32", acc_dtype=acc_dtype)
            for rnd in range(w.rounds):
                _run_round(sh, w, rnd, 0, w.n)
            out[w.name, acc_dtype] = sh
    a, b = out["k2", "f32"], out["k2", "bf16"]
    for name in ("theta", "m", "v"):
        assert np.array_equal(getattr(a, name).view(np.uint32), getattr(b, name).view(np.uint32))
    assert np.array_equal(a.theta_bf16, b.theta_bf16)
    a, b = out["k6", "f32"], out["k6", "bf16"]
    assert not np.array_equal(a.m.view(np.uint32), b.m.view(np.uint32))
    # each rounding of the running sum is at most 2^-9 relative; three adds per stage
    assert np.max(np.abs(a.m - b.m)) <= 3 * 2.0 ** -9 * np.max(np.abs(a.m))
