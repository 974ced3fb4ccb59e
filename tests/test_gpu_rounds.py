"""Whole ACCO rounds on the GPU against the oracle: the five workloads (needs an MI355X).

The tiny workload is compared over the whole shard.  The larger ones run at full size on the
GPU, in the launch configuration the bench uses, and are compared element by element on
sampled index ranges (head, ragged tail, periodic interior blocks): every operation of the
path is elementwise and the inputs are index-addressable, so the oracle computes exactly those
elements.
"""
import time

import numpy as np
import pytest

import oracle
import synth
from parity import (OracleSlices, assert_bf16_close, assert_f32_close, bit_mismatches, bits_of,
                    gather, gpu_run_stage, oracle_warm_state)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def log(*a):
    print(*a, flush=True)


def gpu_hyper(A, w):
    h = w.hyper
    return A.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay)


def run_workload(w: synth.Workload, *, comm_bf16=True, fused=True, warm=None, rounds=None,
                 fused_publish=False, fused_reduce=False, blocked=False, stash=False,
                 bf16_acc=False, schedules=None, adopt=False, batched=False, interleaved=False,
                 comm_block=16384, dev_scalars=False, arena=None):
    import paper_2406_02613_amd as A
    slices = w.sample_slices()
    rounds = w.rounds if rounds is None else rounds
    log(f"workload {w.name}: n={w.n} W={w.workers} rounds={rounds} slices={len(slices)} "
        f"({sum(b - a for a, b in slices)} elements checked)")
    owner = A.ShardOwner(w.n, w.workers, gpu_hyper(A, w), comm_bf16=comm_bf16,
                         fused_bf16_out=fused, fused_publish=fused_publish,
                         fused_reduce=fused_reduce, blocked_state=blocked, bf16_stash=stash,
                         bf16_accumulate=bf16_acc,
                         lr_schedule=None if schedules is None else schedules[0],
                         adopt_first=adopt, batched=batched, interleaved_comm=interleaved,
                         comm_block_elems=comm_block, device_scalars=dev_scalars, arena=arena)
    if warm is None:
        tmp = torch.empty(w.n, dtype=torch.float32, device="cuda")
        w.device_theta(tmp)
        owner.set_state("theta", tmp)
        del tmp
    else:
        for k, name in enumerate(("theta", "m", "v")):
            owner.set_state(name, torch.from_numpy(warm[k]).cuda())
        owner.step.value = w.warm_steps
    grad_buf = torch.empty(w.n, dtype=torch.bfloat16, device="cuda")
    comm = "bf16" if comm_bf16 else "f32"
    acc_dtype = "bf16" if bf16_acc else "f32"
    ref32 = OracleSlices(w, slices, "f32", comm, warm, acc_dtype)
    ref64 = OracleSlices(w, slices, "f64", comm, warm, acc_dtype)
    if schedules is not None:
        for sh in ref32.shards + ref64.shards:
            sh.lr_schedule = schedules[1]
    exact = True
    for r in range(rounds):
        for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
            t0 = time.time()
            gpu_run_stage(owner, w, r, stage, grad_buf, fresh_buffers=adopt)
            torch.cuda.synchronize()
            ref32.run_stage(r, stage)
            ref64.run_stage(r, stage)
            log(f"  round {r} stage {stage}: {time.time() - t0:.1f}s")
            # integer bookkeeping is exact
            table = [w.microbatches(r, k) for k in range(w.workers)]
            if stage == synth.STAGE_TILDE:
                assert owner.total.value == sum(k // 2 for k in table)
                assert owner.step.value == ref32.shards[0].step == (w.warm_steps if warm else 0) + r
                got = bits_of(gather(owner.theta_tilde_bf16, slices))
                w32 = np.concatenate([s.theta_tilde_bf16 for s in ref32.shards])
                w64 = np.concatenate([s.theta_tilde_bf16 for s in ref64.shards])
            else:
                assert owner.total.value == sum(table)
                assert owner.step.value == ref32.shards[0].step == (w.warm_steps if warm else 0) + r + 1
                got = bits_of(gather(owner.theta_bf16, slices))
                w32 = np.concatenate([s.theta_bf16 for s in ref32.shards])
                w64 = np.concatenate([s.theta_bf16 for s in ref64.shards])
            assert_bf16_close(got, w32, f"{w.name} r{r} s{stage} bf16 vs f32 form")
            assert_bf16_close(got, w64, f"{w.name} r{r} s{stage} bf16 vs f64 form")
            exact &= np.array_equal(got, w32)
            if not (fused_reduce and stage == synth.STAGE_FULL):   # fused commit only reads gsum
                gs = gather(owner.get_state("gsum"), slices).numpy()
                assert bit_mismatches(gs, np.concatenate([s.gsum for s in ref32.shards])) == 0
        for name in ("theta", "m", "v"):
            got = gather(owner.get_state(name), slices).numpy()
            a32 = np.concatenate([getattr(s, name) for s in ref32.shards])
            a64 = np.concatenate([getattr(s, name) for s in ref64.shards])
            abs_ = 1e-30 if name == "v" else 1e-9
            assert_f32_close(got, a32, f"{w.name} r{r} {name} vs f32 form", abs_=abs_)
            if name == "theta":
                # independent roundings of two correct implementations add up round by round;
                # scale the relative bound by the largest magnitude theta had, and let the
                # absolute floor grow with the number of Adam steps summed
                ref0 = np.concatenate([w.host_theta(a, b - a) for a, b in slices]) \
                    if warm is None else np.concatenate([warm[0][a:b] for a, b in slices])
                err = np.abs(got.astype(np.float64) - a64)
                bound = np.maximum(1e-9 * max(1, (r + 1) / 2),
                                   2e-6 * np.maximum(np.abs(a64), np.abs(ref0)))
                assert np.all(err <= bound), f"{w.name} r{r} theta vs f64 form"
            else:
                assert_f32_close(got, a64, f"{w.name} r{r} {name} vs f64 form", abs_=abs_)
            exact &= bit_mismatches(got, a32) == 0
    log(f"  bit-exact with the binary32 oracle form over all rounds: {exact}")
    assert exact
    return owner


def test_tiny_three_rounds_whole_shard():
    run_workload(synth.WORKLOADS["tiny"])


def test_tiny_variants_fp32_communication_and_unfused_cast():
    w = synth.WORKLOADS["tiny"]
    run_workload(w, comm_bf16=False, rounds=2)
    run_workload(w, fused=False, rounds=2)


def test_tiny_with_fused_publish_and_fused_reduce():
    w = synth.WORKLOADS["tiny"]
    run_workload(w, fused_publish=True)
    run_workload(w, fused_reduce=True)
    run_workload(w, fused_publish=True, fused_reduce=True)
    run_workload(w, comm_bf16=False, fused_reduce=True, rounds=2)


def test_tiny_with_step_scalars_in_device_memory():
    w = synth.WORKLOADS["tiny"]
    run_workload(w, dev_scalars=True)
    run_workload(w, dev_scalars=True, fused_publish=True, fused_reduce=True, blocked=True,
                 stash=True, batched=True)
    run_workload(w, dev_scalars=True, comm_bf16=False, fused_reduce=True, rounds=2)


def test_tiny_with_bf16_stash():
    w = synth.WORKLOADS["tiny"]
    run_workload(w, stash=True)                                  # one micro-batch per stage
    run_workload(w, stash=True, fused_publish=True, fused_reduce=True, blocked=True)


def test_bf16_running_sums_as_in_the_papers_setup():
    """Accumulators held in bf16 (paper, Sec. 4): different values from the fp32 accumulators,
    and the oracle in the same mode must be met bit for bit."""
    run_workload(synth.WORKLOADS["tiny"], bf16_acc=True)
    w = synth.Workload(name="ragged16", n=300_000 + 37, workers=5, rounds=3, grad_std=1e-3,
                       k_range=(2, 8), zero_frac=0.05, zero_run=64, outlier_frac=1e-2, seed=4)
    run_workload(w, bf16_acc=True)
    run_workload(w, bf16_acc=True, fused_reduce=True, blocked=True)


def test_cosine_learning_rate_schedule_through_the_rounds():
    """The paper's cosine schedule (App. C): the library's host helper on the GPU side, the
    oracle's own on the other; the rate of an update is shared by its two stages."""
    import paper_2406_02613_amd as A
    w = synth.Workload(name="sched", n=200_000 + 5, workers=3, rounds=8, grad_std=1e-3,
                       k_range=(2, 4), seed=6)
    lr = w.hyper.lr
    gpu = lambda t: A.acco_lr_cosine(lr, lr / 10, t, 2, 8)        # noqa: E731
    cpu = lambda t: oracle.lr_cosine(lr, lr / 10, t, 2, 8)        # noqa: E731
    run_workload(w, schedules=(gpu, cpu))
    run_workload(w, schedules=(gpu, cpu), fused_publish=True, fused_reduce=True, blocked=True,
                 stash=True)


def test_first_gradient_adopted_in_place_changes_no_bits():
    """adopt_first: the first micro-batch's buffer serves as the stash where it lies."""
    import paper_2406_02613_amd as A
    w = synth.Workload(name="adopt", n=300_000 + 37, workers=5, rounds=3, grad_std=1e-3,
                       k_range=(2, 8), zero_frac=0.05, zero_run=64, outlier_frac=1e-2, seed=4)
    run_workload(w, stash=True, adopt=True)                       # 1 to 4 micro-batches per stage
    run_workload(w, stash=True, adopt=True, fused_publish=True, fused_reduce=True, blocked=True)
    run_workload(synth.WORKLOADS["tiny"], stash=True, adopt=True, fused_publish=True,
                 fused_reduce=True)                               # one micro-batch per stage
    # reusing the adopted buffer for the next micro-batch is caught
    own = A.ShardOwner(64, 1, gpu_hyper(A, w), bf16_stash=True, adopt_first=True)
    g = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    own.add_microbatch(0, g)
    with pytest.raises(ValueError):
        own.add_microbatch(0, g)


def test_a_stage_without_a_gradient_from_every_worker_is_refused():
    import paper_2406_02613_amd as A
    w = synth.WORKLOADS["tiny"]
    own = A.ShardOwner(256, 2, gpu_hyper(A, w))
    own.add_microbatch(0, torch.zeros(256, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(ValueError):
        own.stage1()
    assert own.step.value == 0 and own.total.value == 0


def test_one_launch_for_all_workers_changes_no_bits():
    """batched: workers at the same step of their accumulation share one launch."""
    tiny = synth.WORKLOADS["tiny"]
    run_workload(tiny, batched=True)                               # base entry points
    run_workload(tiny, batched=True, stash=True, fused_publish=True, fused_reduce=True,
                 blocked=True)
    w = synth.Workload(name="ragged", n=300_000 + 37, workers=5, rounds=3, grad_std=1e-3,
                       k_range=(2, 8), zero_frac=0.05, zero_run=64, outlier_frac=1e-2, seed=4)
    run_workload(w, batched=True)                                  # unequal counts: groups change
    run_workload(w, batched=True, fused_publish=True)
    run_workload(w, batched=True, stash=True)
    run_workload(w, batched=True, stash=True, fused_publish=True, fused_reduce=True, blocked=True)
    run_workload(w, batched=True, stash=True, adopt=True, fused_publish=True, fused_reduce=True)
    run_workload(w, batched=True, bf16_acc=True, fused_reduce=True)
    run_workload(w, batched=True, comm_bf16=False, rounds=2)
    wide = synth.Workload(name="wide", n=70_001, workers=20, rounds=2, grad_std=1e-3,
                          k_range=(2, 5), seed=8)                  # more workers than one launch holds
    run_workload(wide, batched=True, stash=True, fused_publish=True, fused_reduce=True)
    run_workload(wide, batched=True)


def test_interleaved_communication_buffers_change_no_bits():
    """interleaved_comm: the W communication buffers are the interleaved blocks of one buffer."""
    tiny = synth.WORKLOADS["tiny"]
    run_workload(tiny, interleaved=True)                           # base entry points otherwise
    run_workload(tiny, interleaved=True, batched=True, stash=True, fused_publish=True,
                 fused_reduce=True, blocked=True)
    w = synth.Workload(name="ragged", n=300_000 + 37, workers=5, rounds=3, grad_std=1e-3,
                       k_range=(2, 8), zero_frac=0.05, zero_run=64, outlier_frac=1e-2, seed=4)
    run_workload(w, interleaved=True)
    run_workload(w, interleaved=True, comm_block=8, fused_publish=True)
    run_workload(w, interleaved=True, comm_block=4096, batched=True, stash=True)
    run_workload(w, interleaved=True, batched=True, stash=True, fused_publish=True,
                 fused_reduce=True, blocked=True)
    run_workload(w, interleaved=True, comm_block=64, batched=True, stash=True, adopt=True,
                 fused_publish=True, fused_reduce=True)
    wide = synth.Workload(name="wide", n=70_001, workers=20, rounds=2, grad_std=1e-3,
                          k_range=(2, 5), seed=8)                  # more shards than one launch sums
    run_workload(wide, interleaved=True, batched=True, stash=True, fused_publish=True,
                 fused_reduce=True)
    # switching between the two kinds of buffers between rounds keeps the values
    import paper_2406_02613_amd as A
    own = A.ShardOwner(4096 + 5, 2, gpu_hyper(A, tiny), batched=True, interleaved_comm=True,
                       bf16_accumulate=False)
    own.set_options(interleaved_comm=False)
    assert own.comm[0].dim() == 1
    own.set_options(interleaved_comm=True)
    assert own.comm[0].dim() == 2
    with pytest.raises(ValueError):
        A.ShardOwner(64, 2, gpu_hyper(A, tiny), bf16_accumulate=True, interleaved_comm=True)


def test_tiny_with_blocked_state():
    w = synth.WORKLOADS["tiny"]
    run_workload(w, blocked=True)
    run_workload(w, blocked=True, fused_publish=True, fused_reduce=True)


def test_ragged_small_shard_with_unequal_counts():
    w = synth.Workload(name="ragged", n=300_000 + 37, workers=5, rounds=3, grad_std=1e-3,
                       k_range=(2, 8), zero_frac=0.05, zero_run=64, outlier_frac=1e-2, seed=4)
    run_workload(w)
    run_workload(w, fused_publish=True, fused_reduce=True)
    run_workload(w, fused_publish=True, fused_reduce=True, blocked=True)
    run_workload(w, stash=True)                                  # 1 to 4 micro-batches per stage
    run_workload(w, stash=True, fused_publish=True, fused_reduce=True, blocked=True)


def test_gpt2_small_scale_shard_ten_rounds():
    run_workload(synth.WORKLOADS["gpt2s"])


def test_one_billion_scale_shard_warm_state_ten_rounds():
    w = synth.WORKLOADS["1b"]
    t0 = time.time()
    warm = oracle_warm_state(w, 0, w.n)
    log(f"oracle warm state ({w.warm_steps} steps on {w.n} elements): {time.time() - t0:.1f}s")
    assert np.all(warm[2] >= 0) and np.count_nonzero(warm[1]) > 0.99 * w.n
    run_workload(w, warm=warm)


def test_seven_billion_scale_shard_five_rounds():
    run_workload(synth.WORKLOADS["7b"])


def test_seven_billion_heterogeneous_ragged_shard_five_rounds():
    run_workload(synth.WORKLOADS["7b_hetero"])


def test_seven_billion_scale_shard_fused_path_as_benched():
    # the configuration bench.py times by default: bf16 stash, fused publish, fused reduce + step,
    # interleaved state, one accumulate launch for all workers, every buffer of the owner placed
    # by memory class in one arena
    import gc

    import paper_2406_02613_amd as A
    gc.collect()
    torch.cuda.empty_cache()
    free = torch.cuda.mem_get_info()[0]
    arena = None
    if free >= 170 << 30:            # the owner's buffers take 74 GB, the test's own another 20
        arena = A.HbmArena(int(0.75 * free))
        log("arena:", arena.describe())
        if arena.n_classes > 4 or len(arena.runs) > 16 or \
                max(arena.largest_free().values()) < 30 << 30:
            # the classification is a timing measurement; one that was disturbed leaves pieces
            # too small for these buffers.  What this test checks is the arithmetic.
            log("arena too fragmented for the 875M-element buffers: plain allocations")
            arena = None
    else:
        log(f"only {free >> 30} GiB free: plain allocations")
    run_workload(synth.WORKLOADS["7b"], fused_publish=True, fused_reduce=True, blocked=True,
                 stash=True, batched=True, rounds=3, arena=arena)
    del arena
    gc.collect()
    torch.cuda.empty_cache()


def test_seven_billion_hetero_blocked_state_fused_path():
    # ... and with the communication buffers interleaved (bench.py --interleaved-comm)
    run_workload(synth.WORKLOADS["7b_hetero"], fused_publish=True, fused_reduce=True,
                 blocked=True, stash=True, batched=True, interleaved=True, rounds=2)


def test_smaller_workloads_on_the_benched_path():
    for name, rounds in (("gpt2s", 3), ("1b", 2)):
        run_workload(synth.WORKLOADS[name], fused_publish=True, fused_reduce=True, blocked=True,
                     stash=True, batched=True, interleaved=(name == "1b"), rounds=rounds)
