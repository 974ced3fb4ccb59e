"""The AdamW step entry points with their scalars in device memory (the *_dev forms), and whole
rounds recorded once as a HIP graph and replayed while the update index moves on.

What is compared: the *_dev forms with the oracle's binary32 form bit for bit (and thereby with
the by-value forms, which meet the same oracle); recorded rounds with oracle rounds, every replay,
with the owner's eager work and host synchronisations between the replays."""
import numpy as np
import pytest

import oracle
import synth
from parity import OracleSlices, adam_state, bf16_tensor, bit_mismatches, bits_of, gather

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

HP = (6e-4, 0.9, 0.95, 1e-8, 0.1)
HYPER = dict(lr=HP[0], b1=HP[1], b2=HP[2], eps=HP[3], wd=HP[4])


def log(*a):
    print(*a, flush=True)


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _state_tensors(A, arrays, blocked):
    """theta, m, v, gsum on the device, planar or as the components of a blocked buffer."""
    n = arrays[0].size
    if not blocked:
        return None, [_dev(a) for a in arrays]
    st = A.BlockedState(n, 8192, torch.device("cuda"))
    for name, a in zip(("theta", "m", "v", "gsum"), arrays):
        st.load(name, _dev(a))
    return st, [st.theta, st.m, st.v, st.gsum]


def _planar(st, tensors, k):
    return (st.planar(("theta", "m", "v", "gsum")[k]) if st is not None else tensors[k]).cpu().numpy()


@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("n", [5, 70_037, 300_000])
def test_device_scalar_steps_meet_the_oracle_bit_for_bit(n, blocked):
    import paper_2406_02613_amd as A
    B = A.binding
    hp, ohp = A.make_hyper(*HP), oracle.make_hyper(*HP)
    scal = torch.zeros(4 * 16, dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(n + blocked)
    for kind, step, count in (("cold", 0, 1), ("warm", 7, 32), ("wide", 12345, 6)):
        log(f"dev scalars: n={n} blocked={blocked} kind={kind} step={step} count={count}")
        th, m, v, g = adam_state(rng, n, kind, HYPER, step + 1, count)
        # block 2 holds this step's scalars; the blocks around it hold another step's
        B.acco_stage_scalars(scal, [B.acco_fold_adamw(hp, step + 3, count + 1)] * 4, 0)
        B.acco_stage_scalars(scal, [B.acco_fold_adamw(hp, step, count)], 2)

        st, ts = _state_tensors(A, (th, m, v, g), blocked)
        out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
        B.acco_estimate_step_dev(*ts, scal, 2, theta_tilde_bf16=out, n=n)
        _, want16 = oracle.estimate(th, m, v, g, ohp, step + 1, count, want_f32=False,
                                    precision="f32")
        assert np.array_equal(bits_of(out), want16), "estimate_dev"
        for k, a in enumerate((th, m, v, g)):                     # nothing committed
            assert bit_mismatches(_planar(st, ts, k), a) == 0

        th2, m2, v2 = th.copy(), m.copy(), v.copy()
        want16 = oracle.commit(th2, m2, v2, g, ohp, step + 1, count, precision="f32")
        out.zero_()
        B.acco_commit_step_dev(*ts, scal, 2, theta_bf16=out, n=n)
        for k, a in enumerate((th2, m2, v2)):
            assert bit_mismatches(_planar(st, ts, k), a) == 0, ("commit_dev", k)
        assert np.array_equal(bits_of(out), want16), "commit_dev bf16"
        # without the bf16 output
        st, ts = _state_tensors(A, (th, m, v, g), blocked)
        B.acco_commit_step_dev(*ts, scal, 2, n=n)
        for k, a in enumerate((th2, m2, v2)):
            assert bit_mismatches(_planar(st, ts, k), a) == 0, ("commit_dev no out", k)


@pytest.mark.parametrize("W,bf16", [(1, True), (3, True), (9, True), (3, False), (20, True)])
def test_fused_reduce_steps_with_device_scalars(W, bf16):
    import paper_2406_02613_amd as A
    B = A.binding
    n, step = 90_021, 41
    hp, ohp = A.make_hyper(*HP), oracle.make_hyper(*HP)
    rng = np.random.default_rng(100 + W)
    scal = torch.zeros(2 * 16, dtype=torch.float32, device="cuda")
    for blocked in (False, True):
        log(f"fused dev scalars: W={W} bf16={bf16} blocked={blocked}")
        th, m, v, _ = adam_state(rng, n, "warm", HYPER, step + 1, 2 * W)
        acc = [[(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(W)]
               for _ in range(2)]
        shards = [[oracle.cast(a) if bf16 else a for a in half] for half in acc]
        c1, c2 = list(range(1, W + 1)), list(range(2, W + 2))
        t1, t2 = sum(c1), sum(c1) + sum(c2)
        B.acco_stage_scalars(scal, [B.acco_fold_adamw(hp, step, t1),
                                    B.acco_fold_adamw(hp, step, t2)], 0)
        st, ts = _state_tensors(A, (th, m, v, np.zeros(n, np.float32)), blocked)
        out = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
        dev = [[bf16_tensor(s) if bf16 else _dev(s) for s in half] for half in shards]

        gsum = np.empty(n, np.float32)
        oracle.reduce(gsum, shards[0], accumulate_=False)
        _, want16 = oracle.estimate(th, m, v, gsum, ohp, step + 1, t1, want_f32=False,
                                    precision="f32")
        B.acco_reduce_estimate_step_dev(*ts, dev[0], scal, 0, theta_tilde_bf16=out, n=n)
        assert np.array_equal(bits_of(out), want16), "reduce_estimate_dev"
        assert bit_mismatches(_planar(st, ts, 3), gsum) == 0
        for k, a in enumerate((th, m, v)):
            assert bit_mismatches(_planar(st, ts, k), a) == 0

        oracle.reduce(gsum, shards[1], accumulate_=True)
        th2, m2, v2 = th.copy(), m.copy(), v.copy()
        want16 = oracle.commit(th2, m2, v2, gsum, ohp, step + 1, t2, precision="f32")
        out.zero_()
        B.acco_reduce_commit_step_dev(*ts, dev[1], scal, 1, theta_bf16=out, n=n)
        for k, a in enumerate((th2, m2, v2)):
            assert bit_mismatches(_planar(st, ts, k), a) == 0, ("reduce_commit_dev", k)
        assert np.array_equal(bits_of(out), want16)


def _round_buffers(w, rnd):
    """One buffer per micro-batch gradient of a round, by stage and worker."""
    return [[[torch.empty(w.n, dtype=torch.bfloat16, device="cuda") for _ in range(c)]
             for c in w.stage_counts(rnd, stage)] for stage in (synth.STAGE_TILDE, synth.STAGE_FULL)]


def _fill(w, rnd, bufs):
    for si, stage in enumerate((synth.STAGE_TILDE, synth.STAGE_FULL)):
        for wk, row in enumerate(bufs[si]):
            for mb, buf in enumerate(row):
                synth.device_grad_bf16(buf, w.grad_spec(rnd, stage, wk, mb), 0)


def _check_round(owner, ref, slices, what):
    for name in ("theta", "m", "v"):
        got = gather(owner.get_state(name), slices).numpy()
        want = np.concatenate([getattr(s, name) for s in ref.shards])
        assert bit_mismatches(got, want) == 0, (what, name)
    for name in ("theta_bf16", "theta_tilde_bf16"):
        got = bits_of(gather(getattr(owner, name), slices))
        assert np.array_equal(got, np.concatenate([getattr(s, name) for s in ref.shards])), (what, name)
    assert owner.step.value == ref.shards[0].step


@pytest.mark.parametrize("options", [
    dict(fused_publish=True, fused_reduce=True, blocked_state=True, bf16_stash=True, batched=True),
    dict(),
    dict(fused_reduce=True, batched=True, interleaved_comm=True, bf16_stash=True,
         fused_publish=True),
])
def test_recorded_round_replays_follow_the_update_index(options):
    """Round 0 eagerly (device scalars), then the round recorded once and replayed for rounds
    1..5 on new gradients, an eager round in between; with a learning-rate schedule, so that
    every scalar of the two steps changes from replay to replay."""
    import paper_2406_02613_amd as A
    w = synth.Workload(name="rec", n=150_037, workers=3, rounds=7, grad_std=1e-3, k_fixed=4,
                       theta_dist="uniform", theta_param=0.05, seed=5)
    slices = [(0, w.n)]
    sched = (lambda t: A.acco_lr_cosine(6e-4, 6e-5, t, 2, 9),
             lambda t: oracle.lr_cosine(6e-4, 6e-5, t, 2, 9))
    h = w.hyper
    owner = A.ShardOwner(w.n, w.workers, A.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                         device_scalars=True, lr_schedule=sched[0], **options)
    tmp = torch.empty(w.n, dtype=torch.float32, device="cuda")
    w.device_theta(tmp)
    owner.set_state("theta", tmp)
    ref = OracleSlices(w, slices, "f32")
    for sh in ref.shards:
        sh.lr_schedule = sched[1]
    bufs = _round_buffers(w, 0)

    def eager(rnd):
        _fill(w, rnd, bufs)
        owner.add_microbatch_rows(bufs[0])
        owner.stage1()
        owner.add_microbatch_rows(bufs[1])
        owner.stage2()

    def reference(rnd):
        ref.run_stage(rnd, synth.STAGE_TILDE)
        ref.run_stage(rnd, synth.STAGE_FULL)

    log("recorded round: eager round 0", options)
    eager(0)
    reference(0)
    torch.cuda.synchronize()
    _check_round(owner, ref, slices, "eager round 0")

    before = [gather(owner.get_state(k), slices).clone() for k in ("theta", "m", "v")]
    rec = owner.record_round(bufs[0], bufs[1])
    torch.cuda.synchronize()
    assert owner.step.value == 1 and owner.total.value == 4 * w.workers     # as before recording
    for k, b in zip(("theta", "m", "v"), before):                          # no device work
        assert torch.equal(gather(owner.get_state(k), slices).view(torch.int32), b.view(torch.int32))
    assert (rec.total1, rec.total2) == (2 * w.workers, 4 * w.workers)

    for rnd in range(1, 7):
        if rnd == 4:
            log("recorded round: eager round", rnd)
            eager(rnd)
        else:
            log("recorded round: replay for round", rnd)
            _fill(w, rnd, bufs)
            owner.theta_bf16.zero_()
            owner.theta_tilde_bf16.zero_()
            rec.replay()
        reference(rnd)
        torch.cuda.synchronize()
        _check_round(owner, ref, slices, f"round {rnd}")
        assert owner.total.value == 4 * w.workers
        assert [c.value for c in owner.count] == w.stage_counts(rnd, synth.STAGE_FULL)


def test_record_round_refuses_what_it_cannot_replay():
    import paper_2406_02613_amd as A
    n, W = 4096, 2
    hp = A.make_hyper(*HP)
    g = [[torch.zeros(n, dtype=torch.bfloat16, device="cuda")] for _ in range(W)]
    plain = A.ShardOwner(n, W, hp)
    with pytest.raises(ValueError):
        plain.record_round(g, g)
    owner = A.ShardOwner(n, W, hp, device_scalars=True)
    with pytest.raises(ValueError):
        owner.record_round(g[:1], g)
    owner.add_microbatch(0, g[0][0])
    with pytest.raises(ValueError):
        owner.record_round(g, g)
