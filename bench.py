#!/usr/bin/env python3
"""Benchmark of the ACCO per-shard optimizer path on one MI355X.

A step is one ACCO round of one shard owner, sequenced by paper_2406_02613_amd.ShardOwner (the
same object the parity tests drive): every micro-batch gradient of every simulated worker is
accumulated, each worker's sum is published to its bf16 communication buffer, the owner reduces
the W buffers and runs the speculative estimate step, then the second half is accumulated,
published and reduced onto the retained sum and the committed AdamW step runs with its fused
bf16 parameter output.  All inputs (parameters, optimizer state, every micro-batch gradient of
the round) are resident in HBM before the timed region starts.  By default every buffer comes
from one arena in which the owner's buffers and the gradients are placed by memory class of the
HBM (paper_2406_02613_amd.arena; `--no-arena` for plain allocations); config.placement says
which it was.

Prints ONE JSON line.
  value        shard elements per second through one whole round
  kernels      every kernel of the timed round, timed with HIP events on the launching stream
  roofline     acco_commit_step (fused bf16 output) on its own, on the same buffers after the
               timed region, at the workload's shard length and - for the two 875M-element
               workloads - at both 875,000,000 and 875,000,037 elements; `in_timed_round`
               inside it is the committed-step kernel of the timed round itself (the fused
               reduce + commit)
  checked      after the timed region the state (theta, m, v, both bf16 outputs) on sampled
               index ranges is compared bit for bit with the CPU oracle's binary32 form replayed
               for the same number of rounds on the same gradients
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload on this machine

`bench.py --summarize-rocprof DIR` runs no GPU work: it formats rocprofv3 output found under DIR
(kernel statistics, FETCH_SIZE / WRITE_SIZE counters) into the text summaries kept under
profiles/.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E peak, GB/s
HEADLINE_SIZES = (875_000_000, 875_000_037)   # the two shard lengths the bandwidth bar is set on


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b",
                    help="tiny | gpt2s | 1b | 7b | 7b_hetero (default: the 875M-element shard)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true",
                    help="skip the comparison of the timed state with the oracle")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the base-entry-point round, the adopted-gradient round and the "
                         "bandwidth probes (the headline step kernels are still timed)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="target CPU time of the oracle sample")
    ap.add_argument("--scheme", default=None, choices=["acco", "ddp", "dpu", "wp"],
                    help="time one round of this update scheme sequenced on the base entry "
                         "points (paper_2406_02613_amd.schemes) instead of the default fused "
                         "ACCO round; the JSON line then carries that scheme's round time")
    ap.add_argument("--two-stream", action="store_true",
                    help="run the two-stream scheduler of Alg. 1 (computation stream accumulating "
                         "while the communication stream runs the owner's stage) and report what "
                         "the overlap costs each stream")
    ap.add_argument("--link-ms", type=float, default=0.0,
                    help="--two-stream: a timed wait of this many ms per stage on the "
                         "communication stream where the reduce-scatter / all-gather transfers "
                         "would be (no data moves; it only occupies the stream)")
    ap.add_argument("--gemm", type=int, default=8192,
                    help="--two-stream: size of the square bf16 GEMM standing in for a "
                         "micro-batch's forward/backward (0 = none)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the shard (fp32, n elements read and "
                         "n written) so that a counter run has a kernel of known traffic")
    ap.add_argument("--planar-state", action="store_true",
                    help="theta, m, v, gsum as four separate planar arrays instead of the "
                         "block-interleaved state buffer")
    ap.add_argument("--block-elems", type=int, default=8192,
                    help="elements per block of the interleaved state buffer")
    ap.add_argument("--unfused-cast", action="store_true",
                    help="commit without the fused bf16 output, then acco_cast_params")
    ap.add_argument("--unfused-publish", action="store_true",
                    help="publish with acco_cast_params instead of acco_accumulate_publish")
    ap.add_argument("--no-bf16-stash", action="store_true",
                    help="expand the first micro-batch to the fp32 accumulator (acco_accumulate "
                         "init) instead of keeping it as a bf16 stash")
    ap.add_argument("--bf16-accumulate", action="store_true",
                    help="running sums held in bf16 as in the paper's own setup "
                         "(acco_accumulate_bf16; the accumulator is the communication buffer). "
                         "Changes the values: the sum is rounded after every micro-batch")
    ap.add_argument("--unfused-reduce", action="store_true",
                    help="acco_reduce_shards + acco_estimate/commit_step instead of the fused "
                         "reduce+step entry points")
    ap.add_argument("--base-path", action="store_true",
                    help="the five base entry points only (= all three --unfused-* flags "
                         "except the fused bf16 output of the commit)")
    ap.add_argument("--interleaved-comm", action="store_true",
                    help="the W communication buffers as the interleaved blocks of one buffer "
                         "instead of W separate ones (same values; the reduce kernels get faster "
                         "and steadier, the publishing kernels slower)")
    ap.add_argument("--comm-block-elems", type=int, default=16384,
                    help="elements per block of the interleaved communication buffers")
    ap.add_argument("--no-arena", action="store_true",
                    help="plain allocations instead of one arena with the buffers placed by "
                         "memory class (what the kernels read together in one class of the HBM, "
                         "their outputs in another)")
    ap.add_argument("--per-worker-launches", action="store_true",
                    help="one accumulate launch per worker and micro-batch instead of one launch "
                         "for all workers that are at the same point of their accumulation")
    ap.add_argument("--summarize-rocprof", metavar="DIR", default=None,
                    help="no GPU work: format the rocprofv3 output under DIR (DIR/trace, "
                         "DIR/fetch, DIR/write and the bench lines DIR/*.json written by the "
                         "profiled runs) into profiles/bench_<workload>_*.txt")
    return ap.parse_args()


PAPER_CONTEXT = {
    "what": "end-to-end training wall-clock, ZeRO-1 (DDP + sharded optimizer) vs ACCO; the paper "
            "gives no time, GB/s or elements/s for the shard optimizer path measured here",
    "pretrain_GPT-Neo-125M_6B_tokens_1x8_H100-PCIe": {"zero1": "4h41m", "acco": "4h25m"},
    "pretrain_GPT-Neo-125M_50B_tokens_4x8_A100-80GB": {"zero1": "14h41m", "acco": "10h55m"},
    "finetune_GPT-Neo-2.7B_80M_tokens_1x8_A100-80GB": {"zero1": "43min", "acco": "25min"},
    "finetune_GPT-Neo-2.7B_80M_tokens_2x4_A100-80GB": {"zero1": "3h46m", "acco": "29min"},
    "source": "paper, table of training times (pre-training and fine-tuning), Sec. 4",
}


class EventLog:
    """HIP event pairs on torch's current stream (the stream every kernel is launched on).
    An instance is what ShardOwner.trace takes: log(label, fn, *args) runs fn between two events."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = {}      # label -> list of (start, end)
        self.enabled = False

    def __call__(self, name, fn, *a, **kw):
        if not self.enabled:
            return fn(*a, **kw)
        s = self.torch.cuda.Event(enable_timing=True)
        e = self.torch.cuda.Event(enable_timing=True)
        s.record()
        out = fn(*a, **kw)
        e.record()
        self.pairs.setdefault(name, []).append((s, e))
        return out

    def summary(self):
        return {k: [s.elapsed_time(e) for s, e in v] for k, v in self.pairs.items()}


def run_round(owner, w, grads):
    """One ACCO round of the shard owner on resident gradients grads[stage][worker][mb]."""
    import synth
    for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
        rows = grads[stage]
        owner.add_microbatch_rows(rows)
        if stage == synth.STAGE_TILDE:
            owner.stage1()
        else:
            owner.stage2()


def kernel_bytes_per_elem(name, workers):
    """Algorithmic HBM bytes per shard element of one launch (per worker for the batched
    accumulation launches, whose labels end in the number of workers they cover)."""
    from paper_2406_02613_amd import layout
    red = 2 * workers                              # W bf16 shards read
    table = {
        "reduce_init": red + 4, "reduce_accumulate": red + 8,
        "accumulate_publish": 4 + 2 + 2,           # acc read, grad read, bf16 comm written
        "accumulate_publish_init": 2 + 2,
        "accumulate_bf16_init": 2 + 2,             # grad read, bf16 running sum written
        "accumulate_bf16": 2 + 2 + 2,              # running sum and grad read, sum written
        "accumulate_first": 2 + 2,                 # grad read, bf16 stash written
        "accumulate_first_publish": 2 + 2,
        "accumulate_second": 2 + 2 + 4,            # stash, grad read; fp32 acc written
        "accumulate_second_publish": 2 + 2 + 2,    # stash, grad read; bf16 comm written
        "reduce_estimate": 12 + red + 4 + 2,       # theta,m,v + shards read; gsum, bf16 written
        "reduce_commit": 12 + 4 + red + 12,        # theta,m,v,gsum + shards read; theta,m,v written
        "reduce_commit_bf16": 12 + 4 + red + 12 + 2,
    }
    name = name.replace("@dev", "")                # the device-scalar form moves the same bytes
    if "*" in name:                                # "label*k": one launch over k workers
        base, k = name.split("*")
        return int(k) * kernel_bytes_per_elem(base, workers)
    return table[name] if name in table else layout.BYTES_PER_ELEM[name]


def scheme_round(owner, w, grads):
    """One round of owner.scheme on resident gradients (base entry points, unfused)."""
    import synth
    for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
        for wk in range(w.workers):
            for g in grads[stage][wk]:
                owner.add_microbatch(wk, g)
        if stage == synth.STAGE_TILDE and owner.scheme == "acco":
            owner.finish_half()
    owner.finish_round()


def small_arena(args, torch, A):
    """An arena for the side benches (two-stream, schemes), or None: --no-arena, too little
    memory, or timings too erratic to classify by."""
    if args.no_arena:
        return None
    try:
        arena = A.HbmArena(min(int(0.7 * torch.cuda.mem_get_info()[0]), 200 << 30))
    except (A.AccoError, MemoryError, RuntimeError, ValueError) as e:
        print(f"bench.py: no arena ({e}); plain allocations", file=sys.stderr)
        return None
    return None if arena.n_classes > 4 or len(arena.runs) > 16 else arena


def bench_scheme(args, torch, A, w, synth):
    h = w.hyper
    arena = small_arena(args, torch, A)
    owner = A.SchemeOwner(w.n, w.workers, args.scheme,
                          A.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                          arena=arena)
    grads = make_grads(torch, synth, w, owner if arena is not None else None, hint_first=False)[0]
    tmp = torch.empty(w.n, dtype=torch.float32, device="cuda")
    w.device_theta(tmp)
    owner.set_theta(tmp)
    del tmp
    for _ in range(args.warmup):
        scheme_round(owner, w, grads)
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(args.steps):
        scheme_round(owner, w, grads)
    e.record()
    torch.cuda.synchronize()
    ms = s.elapsed_time(e) / args.steps
    print(json.dumps({
        "metric": f"shard optimizer-step elements/s (one round of scheme '{args.scheme}', "
                  "base entry points)",
        "value": w.n / (ms * 1e-3), "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "scheme": args.scheme, "n": w.n, "workers": w.workers,
                   "placement": ("one arena, buffers placed by memory class: " + arena.describe()
                                 if arena is not None else "plain allocations")}}))
    return 0


def bench_two_stream(args, torch, A, w):
    """Alg. 1's two streams on one GPU at the workload's shard size: worker 0 accumulates on the
    computation stream (GEMM stand-in + gradient write + acco_accumulate per micro-batch) while
    the communication stream publishes, reduces over W shards and runs the estimate / commit."""
    import synth
    h = w.hyper
    arena = small_arena(args, torch, A)
    own = A.TwoStreamOwner(w.n, w.workers, A.make_hyper(h.lr, h.beta1, h.beta2, h.eps,
                                                        h.weight_decay), arena=arena)
    tmp = torch.empty(w.n, dtype=torch.float32, device="cuda")
    w.device_theta(tmp)
    own.set_theta(tmp)
    del tmp
    peers = []
    for wk in range(1, w.workers):
        p = own.new_peer_buffer(wk)
        synth.device_grad_bf16(p, w.grad_spec(0, 1, wk, 0), 0)
        peers.append(p)
    peer_counts = [2] * (w.workers - 1)
    buf = own.new_buffer("compute", w.n, torch.bfloat16)
    a = b = None
    if args.gemm > 0:
        a = torch.randn(args.gemm, args.gemm, dtype=torch.bfloat16, device="cuda")
        b = torch.randn(args.gemm, args.gemm, dtype=torch.bfloat16, device="cuda")
    c = torch.empty(args.gemm, args.gemm, dtype=torch.bfloat16, device="cuda") if a is not None \
        else None

    def compute():
        if a is not None:
            torch.mm(a, b, out=c)

    def grad_source(rnd, acc, k):
        synth.device_grad_bf16(buf, w.grad_spec((rnd + 1) & 0xFFFF, acc, 0, k & 0xFFFF), 0)
        return buf

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    # each stream on its own first
    def one_microbatch():
        compute()
        B = A.binding
        B.acco_accumulate(own.acc[2], grad_source(0, 2, 0), False)
    own.acc[2].zero_()
    mb_alone = timed(one_microbatch, 10)

    def comm_pair():
        own._communicate(1, peers, peer_counts)
        own._communicate(2, peers, peer_counts)
        own.comm_stream.synchronize()
    own.count[1].value = own.count[2].value = 2
    comm_alone = timed(comm_pair, 5) / 2
    own.step.value = 0

    transport = None
    if args.link_ms > 0:
        # calibrate torch's spin kernel (cycles per ms) once, then wait link_ms per stage
        probe = 20_000_000
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda._sleep(1000)
        e0.record()
        torch.cuda._sleep(probe)
        e1.record()
        torch.cuda.synchronize()
        cycles = int(args.link_ms * probe / e0.elapsed_time(e1))
        transport = lambda: torch.cuda._sleep(cycles)

    own.run(args.warmup, grad_source, peers, peer_counts, compute, transport=transport)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    log = own.run(args.steps, grad_source, peers, peer_counts, compute, transport=transport)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    st1 = [r for r in log.stages if r.stage == 1]
    st2 = [r for r in log.stages if r.stage == 2]
    mbs = sum(r.microbatches for r in log.stages)
    mean = lambda xs: sum(xs) / max(len(xs), 1)
    out = {
        "metric": "shard optimizer-step elements/s (two-stream ACCO round: communication stream "
                  "overlapped with gradient accumulation)",
        "value": w.n * args.steps / (wall_ms * 1e-3), "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_ms / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "mode": "two-stream", "n": w.n, "workers": w.workers,
                   "gemm": args.gemm, "link_ms_per_stage": args.link_ms,
                   "placement": ("one arena, buffers placed by memory class: " + arena.describe()
                                 if arena is not None else "plain allocations")},
        "two_stream": {
            "microbatch_ms_alone": mb_alone,
            "microbatch_ms_overlapped": mean([r.comp_ms / r.microbatches for r in log.stages]),
            "comm_stage_ms_alone": comm_alone,
            "comm_stage1_ms_overlapped": mean([r.comm_ms for r in st1]),
            "comm_stage2_ms_overlapped": mean([r.comm_ms for r in st2]),
            "microbatches_per_stage": mean([r.microbatches for r in log.stages]),
            "supplementary_accumulation_steps": log.extra_accumulations(1),
            "microbatches_total": mbs,
        },
    }
    print(json.dumps(out))
    return 0


def cpu_baseline(w, target_seconds, acc_dtype="f32"):
    """The oracle (as it stands) on the first S elements of the same workload, one round."""
    import numpy as np
    import oracle
    import synth
    cores = min(oracle.usable_cores(), 64)
    oracle.set_threads(cores)
    h = w.hyper
    hp = oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay)

    def rounds(S, R):
        """R rounds on the first S elements; inputs are generated outside the timed region."""
        grads = {st: [[synth.host_grad_bf16(w.grad_spec(0, st, wk, mb), 0, S)
                       for mb in range(w.stage_counts(0, st)[wk])] for wk in range(w.workers)]
                 for st in (synth.STAGE_TILDE, synth.STAGE_FULL)}
        sh = oracle.OracleShard(w.host_theta(0, S), w.workers, hp, precision="f64",
                                acc_dtype=acc_dtype)
        t0 = time.perf_counter()
        for _ in range(R):
            for st in (synth.STAGE_TILDE, synth.STAGE_FULL):
                for wk in range(w.workers):
                    for g in grads[st][wk]:
                        sh.add_microbatch(wk, g)
                if st == synth.STAGE_TILDE:
                    sh.stage1()
                else:
                    sh.stage2()
        return time.perf_counter() - t0

    def commit_alone(S, R):
        rng = np.random.default_rng(0)
        th = w.host_theta(0, S)
        m = np.zeros(S, np.float32)
        v = np.zeros(S, np.float32)
        g = (rng.standard_normal(S) * w.grad_std).astype(np.float32)
        oracle.commit(th, m, v, g, hp, 1, 1, want_bf16=True)
        t0 = time.perf_counter()
        for r in range(R):
            oracle.commit(th, m, v, g, hp, r + 2, 32, want_bf16=True)
        return time.perf_counter() - t0

    S = int(min(w.n, 1 << 24))            # ~100 host bytes per sampled element
    rounds(min(S, 1 << 18), 1)            # page in, start the thread pool
    t1 = rounds(S, 1)
    R = int(max(1, min(200, round(0.6 * target_seconds / max(t1, 1e-6)))))
    t = rounds(S, R)
    tc = commit_alone(S, 20)
    # the same oracle on one thread, on a smaller sample (about a fifth of the time budget)
    oracle.set_threads(1)
    S1 = int(min(S, 1 << 21))
    t11 = rounds(S1, 1)
    R1 = int(max(1, min(50, round(0.2 * target_seconds / max(t11, 1e-6)))))
    ts = rounds(S1, R1)
    tc1 = commit_alone(S1, 10)
    oracle.set_threads(cores)
    return {"value": S * R / t, "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": f"{R} full rounds of workload '{w.name}' on its first {S} shard elements "
                      f"(binary64 form, {cores} OpenMP threads, {t:.1f} s)",
            "commit_step_alone_elements_per_s": S * 20 / tc,
            "single_thread": {"value": S1 * R1 / ts, "cores": 1,
                              "commit_step_alone_elements_per_s": S1 * 10 / tc1,
                              "sample": f"{R1} rounds on the first {S1} elements, {ts:.1f} s"}}


# ------------------------------------------------------------------ rocprofv3 summaries

# kernel-name fragment -> label of bench.py's kernel table ("*" = one launch over several workers)
KERNEL_LABELS = (
    ("Batch<acco::StashOp<false,", "accumulate_first*"),
    ("Batch<acco::StashOp<true,", "accumulate_first_publish*"),
    ("Batch<acco::SecondPublishOp<", "accumulate_second_publish*"),
    ("Batch<acco::SecondOp", "accumulate_second*"),
    ("Batch<acco::AccumulateOp<true>", "accumulate_init*"),
    ("Batch<acco::AccumulateOp<false>", "accumulate*"),
    ("Batch<acco::AccumulatePublishOp<false, false,", "accumulate_publish*"),
    ("Batch<acco::CastOp<", "cast*"),
    ("Single<acco::StashOp<false,", "accumulate_first"),
    ("Single<acco::StashOp<true,", "accumulate_first_publish"),
    ("Single<acco::SecondPublishOp<", "accumulate_second_publish"),
    ("Single<acco::SecondOp", "accumulate_second"),
    ("Single<acco::AccumulateOp<true>", "accumulate_init"),
    ("Single<acco::AccumulateOp<false>", "accumulate"),
    ("Single<acco::AccumulatePublishOp<false, false,", "accumulate_publish"),
    ("Single<acco::AccumulatePublishOp<true, false,", "accumulate_publish_init"),
    ("Single<acco::CastOp<", "cast"),
    ("ReduceAdamOp<false, true, false, true, false, true", "reduce_estimate"),
    ("ReduceAdamOp<true, true, true, false, false, true", "reduce_commit_bf16"),
    ("ReduceAdamOp<true, true, true, false, false, false", "reduce_commit"),
    ("Single<acco::AdamOp<true, false, true", "commit_bf16"),
    ("Single<acco::AdamOp<true, false, false", "commit"),
    ("Single<acco::AdamOp<false, false, true", "estimate"),
    ("ReduceOp<8, true, false", "reduce_init"),
    ("ReduceOp<8, true, true", "reduce_accumulate"),
    ("ReduceOp<16, true, false", "reduce_init"),              # more than 8 bf16 shards
    ("ReduceOp<16, true, true", "reduce_accumulate"),
)


def _short_kernel(name):
    import re
    name = name.replace("void acco::flat_kernel<acco::", "").replace("void acco::stream_kernel<", "")
    name = name.replace("(anonymous namespace)::", "").replace("acco::", "")
    return re.sub(r" ?>?\(.*$", "", name)


def _label_of(kernel_name, grid_size, n):
    """bench label of a dispatch; batched launches get their worker count from the grid."""
    for frag, label in KERNEL_LABELS:
        if frag in kernel_name:
            if "ScalarsFromDevice" in kernel_name:            # the *_dev form of a step kernel
                return label + "@dev"
            if label.endswith("*"):
                per_lane = 8 if ("StashOp" in frag or "SecondPublishOp" in frag) else 4
                one = -(-(n // per_lane) // 64) * 64          # work-items of one worker's row
                return label + str(max(1, round(grid_size / one)))
            return label
    return None


def summarize_rocprof(raw):
    """Text summaries under profiles/ from rocprofv3 output.  For every bench line raw/TAG.json:
    raw/TAG/*_kernel_stats.csv (a --kernel-trace --stats run of the command in raw/TAG.cmd) ->
    profiles/TAG_kernel_stats.txt; raw/TAG_fetch and raw/TAG_write (--pmc FETCH_SIZE /
    WRITE_SIZE runs with --calibrate-copy) -> profiles/TAG_hbm_traffic.txt."""
    import collections
    import csv
    import glob
    wrote = []
    for jpath in sorted(glob.glob(os.path.join(raw, "*.json"))):
        tag = os.path.basename(jpath)[:-5]
        try:
            line = json.loads(open(jpath).read().strip().splitlines()[-1])
        except (ValueError, IndexError):
            continue
        cfg = line.get("config", {})
        n, workers = cfg.get("n"), cfg.get("workers")
        cmd = lambda t: (open(os.path.join(raw, t + ".cmd")).read().strip()    # noqa: E731
                         if os.path.exists(os.path.join(raw, t + ".cmd")) else "(not recorded)")
        stats = glob.glob(os.path.join(raw, tag, "*_kernel_stats.csv"))
        if stats:
            out = [f"rocprofv3 kernel statistics - {line.get('metric', '')}",
                   f"workload: {cfg.get('workload', '?')}", "",
                   "Command (from /tmp with TMPDIR=/tmp on the MI355X box; $R = repository root):",
                   "  " + cmd(tag), "",
                   f"{'kernel':96s} {'calls':>6s} {'avg_ns':>10s} {'min_ns':>10s} {'max_ns':>10s} {'%':>6s}"]
            rows = list(csv.DictReader(open(stats[0])))
            for r in rows[:28]:
                out.append(f"{_short_kernel(r['Name'])[:96]:96s} {r['Calls']:>6s} "
                           f"{float(r['AverageNs']):10.0f} {r['MinNs']:>10s} {r['MaxNs']:>10s} "
                           f"{float(r['Percentage']):6.2f}")
            ks = line.get("kernels")
            if isinstance(ks, dict) and n:
                out += ["", "Same run, bench.py's own HIP-event timing (timed rounds only):"]
                for k, v in ks.items():
                    out.append(f"  {k:30s} {v['calls_per_step']:5.1f} calls/round  avg {v['avg_ms']:.4f} ms"
                               f"  {v['bytes_per_elem']:3d} B/elem  {v['GB/s']:7.1f} GB/s  "
                               f"{100 * v['frac_of_peak']:.1f} % of 8 TB/s")
                out.append(f"  whole round: {line['ms_per_step']:.3f} ms -> {line['value']:.4g} shard "
                           f"elements/s; checked against the oracle: {line.get('checked')}")
                # rocprofv3's own durations against the events', kernel by kernel (from the
                # per-dispatch trace, where a batched launch shows its worker count as grid.y)
                tr = glob.glob(os.path.join(raw, tag, "*_kernel_trace.csv"))
                if tr:
                    dur = collections.defaultdict(list)
                    for r in csv.DictReader(open(tr[0])):
                        lab = _label_of(r["Kernel_Name"], 0, n)
                        if lab:
                            if "*" in lab:
                                lab = lab.split("*")[0] + "*" + r["Grid_Size_Y"]
                            dur[lab].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
                    out += ["", "Agreement of the two clocks (rocprofv3: average over ALL launches of that "
                                "kernel and worker count in the process; events: the timed rounds):"]
                    for k, v in ks.items():
                        if k in dur:
                            out.append(f"  {k:30s} rocprofv3 {sum(dur[k]) / len(dur[k]) / 1e6:.4f} ms "
                                       f"({len(dur[k])} launches)   events {v['avg_ms']:.4f} ms")
            sa = line.get("standalone_step_kernels")
            if isinstance(sa, dict):
                out += ["", "acco_commit_step / acco_estimate_step on their own after the timed region "
                            "(HIP events), per shard length:"]
                for n_k, tab in sa.items():
                    for k, v in tab.items():
                        out.append(f"  n={n_k:>11s} {k:12s} avg {v['avg_ms']:.4f} ms  {v['bytes_per_elem']:2d} B/elem"
                                   f"  {v['GB/s']:7.1f} GB/s  {100 * v['frac_of_peak']:.1f} % of 8 TB/s")
            for key in ("two_stream", "base_entry_points_round", "adopted_first_gradient_round",
                        "recorded_graph_round"):
                if isinstance(line.get(key), dict):
                    out += ["", f"{key}: " + json.dumps({k: v for k, v in line[key].items()
                                                         if k != "kernels"})]
            path = os.path.join(ROOT, "profiles", f"{tag}_kernel_stats.txt")
            open(path, "w").write("\n".join(out) + "\n")
            wrote.append(path)
        fetch = glob.glob(os.path.join(raw, tag + "_fetch", "*_counter_collection.csv"))
        write = glob.glob(os.path.join(raw, tag + "_write", "*_counter_collection.csv"))
        if fetch and write and n:
            vals = collections.defaultdict(lambda: {"FETCH_SIZE": [], "WRITE_SIZE": []})
            names = {}
            copies = {"FETCH_SIZE": [], "WRITE_SIZE": []}
            for ctr, f in (("FETCH_SIZE", fetch[0]), ("WRITE_SIZE", write[0])):
                for r in csv.DictReader(open(f)):
                    if "copyBuffer" in r["Kernel_Name"]:
                        copies[ctr].append(float(r["Counter_Value"]))
                        continue
                    lab = _label_of(r["Kernel_Name"], int(r["Grid_Size"]), n)
                    if lab:
                        vals[lab][ctr].append(float(r["Counter_Value"]))
                        names[lab] = _short_kernel(r["Kernel_Name"])
            if not copies["FETCH_SIZE"] or not copies["WRITE_SIZE"]:
                continue
            # the calibration copy is the large one (torch also issues tiny copies)
            fs = 4.0 * n / (max(copies["FETCH_SIZE"]) * 1024)
            ws = 4.0 * n / (max(copies["WRITE_SIZE"]) * 1024)
            out = [f"HBM traffic per launch from rocprofv3 counters - workload: {cfg.get('workload', '?')}",
                   "", "Commands (from /tmp with TMPDIR=/tmp; one counter per run; $R = repository root):",
                   "  " + cmd(tag + "_fetch"), "  " + cmd(tag + "_write"), "",
                   "Calibration: --calibrate-copy issues one plain device copy of n fp32 (4 n bytes read, "
                   "4 n written;", f"it runs as __amd_rocclr_copyBuffer).  FETCH_SIZE reads "
                   f"{max(copies['FETCH_SIZE']):.1f} KiB for it, WRITE_SIZE {max(copies['WRITE_SIZE']):.1f} KiB,",
                   f"so FETCH_SIZE is scaled by {fs:.3f} and WRITE_SIZE by {ws:.3f} to give bytes.", "",
                   f"{'bench label':30s} {'kernel':44s} {'launches':>8s} {'FETCH KiB':>12s} {'WRITE KiB':>12s} "
                   f"{'read B/el':>9s} {'write B/el':>10s} {'total':>7s} {'algorithmic':>11s}"]
            table = {}
            for lab, v in sorted(vals.items()):
                if not v["FETCH_SIZE"] or not v["WRITE_SIZE"]:
                    continue
                f = sum(v["FETCH_SIZE"]) / len(v["FETCH_SIZE"])
                wv = sum(v["WRITE_SIZE"]) / len(v["WRITE_SIZE"])
                rb, wb = f * 1024 * fs / n, wv * 1024 * ws / n
                table[lab] = round(rb + wb, 3)
                out.append(f"{lab:30s} {names[lab][:44]:44s} {len(v['FETCH_SIZE']):8d} {f:12.1f} {wv:12.1f} "
                           f"{rb:9.3f} {wb:10.3f} {rb + wb:7.2f} {kernel_bytes_per_elem(lab, workers):11d}")
            out += ["", "B/el = bytes per shard element per launch (a launch over k workers moves k workers' "
                        "bytes).", "Measured traffic equals the algorithmic bytes where the last two columns agree.",
                    "", "TRAFFIC_B_PER_ELEM_JSON " + json.dumps(table)]
            path = os.path.join(ROOT, "profiles", f"{tag}_hbm_traffic.txt")
            open(path, "w").write("\n".join(out) + "\n")
            wrote.append(path)
    for pth in wrote:
        print("wrote", os.path.relpath(pth, ROOT))
    return 0 if wrote else 1


def make_grads(torch, synth, w, owner=None, hint_first=True):
    """Every micro-batch gradient of one round, resident in HBM: grads[stage][worker][mb].
    With an owner that places its buffers (an arena), the gradients come from it too."""
    grads = {}
    n_bufs = 0
    for st in (synth.STAGE_TILDE, synth.STAGE_FULL):
        grads[st] = []
        for wk in range(w.workers):
            row = []
            for mb in range(w.stage_counts(0, st)[wk]):
                g = (torch.empty(w.n, dtype=torch.bfloat16, device="cuda") if owner is None
                     else owner.new_gradient_buffer(first=(mb == 0)) if hint_first
                     else owner.new_gradient_buffer())
                synth.device_grad_bf16(g, w.grad_spec(0, st, wk, mb), 0)
                row.append(g)
                n_bufs += 1
            grads[st].append(row)
    torch.cuda.synchronize()
    return grads, n_bufs


class OracleReplay:
    """The checker leg: the CPU oracle (binary32 form) on sampled index ranges of the workload,
    fed the same gradients round after round, to be compared with what the GPU holds."""

    ARRAYS = ("theta", "m", "v", "theta_bf16", "theta_tilde_bf16")

    def __init__(self, w, acc_dtype="f32"):
        import oracle
        import synth
        self.w, self.slices = w, w.sample_slices()
        h = w.hyper
        hp = oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay)
        self.shards = [oracle.OracleShard(w.host_theta(a, b - a), w.workers, hp, precision="f32",
                                          acc_dtype=acc_dtype) for a, b in self.slices]
        self.grads = [{st: [[synth.host_grad_bf16(w.grad_spec(0, st, wk, mb), a, b - a)
                             for mb in range(w.stage_counts(0, st)[wk])]
                            for wk in range(w.workers)]
                       for st in (synth.STAGE_TILDE, synth.STAGE_FULL)} for a, b in self.slices]
        self.rounds = 0

    def run(self, rounds):
        import synth
        for sh, gr in zip(self.shards, self.grads):
            for _ in range(rounds):
                for st in (synth.STAGE_TILDE, synth.STAGE_FULL):
                    for wk, row in enumerate(gr[st]):
                        for g in row:
                            sh.add_microbatch(wk, g)
                    sh.stage1() if st == synth.STAGE_TILDE else sh.stage2()
        self.rounds += rounds

    def snapshot(self, torch, owner):
        """Host copies of the GPU's arrays on the sampled ranges (taken outside any timed region)."""
        snap = {}
        for name in ("theta", "m", "v"):
            full = owner.get_state(name)
            snap[name] = torch.cat([full[a:b] for a, b in self.slices]).cpu().numpy()
            del full
        for name in ("theta_bf16", "theta_tilde_bf16"):
            t = getattr(owner, name)
            snap[name] = torch.cat([t[a:b] for a, b in self.slices]).view(torch.int16).cpu().numpy()
        snap["step"] = owner.step.value
        return snap

    def compare(self, snap):
        """Bit-for-bit comparison of a snapshot with the oracle's present state."""
        import numpy as np
        bad = {}
        for name in self.ARRAYS:
            want = np.concatenate([getattr(sh, name) for sh in self.shards])
            got = snap[name]
            if name.endswith("bf16"):
                diff = got.view(np.uint16) != want.view(np.uint16)
            else:
                diff = got.view(np.uint32) != want.view(np.uint32)
            if diff.any():
                bad[name] = int(diff.sum())
        if snap["step"] != self.shards[0].step:
            bad["step"] = (snap["step"], self.shards[0].step)
        elems = sum(b - a for a, b in self.slices)
        return {"ok": not bad, "mismatches": bad, "elements": elems, "rounds": self.rounds,
                "ranges": len(self.slices)}


def time_rounds(torch, owner, w, grads, reps, warm=1):
    """A few more rounds with the owner's present options, per-kernel events included."""
    log = EventLog(torch)
    owner.trace = log
    for _ in range(warm):
        run_round(owner, w, grads)
    log.enabled = True
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run_round(owner, w, grads)
    e1.record()
    torch.cuda.synchronize()
    owner.trace = None
    ms = e0.elapsed_time(e1) / reps
    summ = log.summary()
    bpe = sum(kernel_bytes_per_elem(k, w.workers) * len(v) / reps for k, v in summ.items())
    return {"ms_per_step": round(ms, 4), "steps": reps, "elements/s": w.n / (ms * 1e-3),
            "bytes_per_elem": bpe, "GB/s": round(bpe * w.n / (ms * 1e-3) / 1e9, 1),
            "launches_per_step": sum(len(v) for v in summ.values()) / reps,
            "kernels": {k: {"calls_per_step": len(v) / reps, "avg_ms": round(sum(v) / len(v), 4),
                            "GB/s": round(kernel_bytes_per_elem(k, w.workers) * w.n
                                          / (sum(v) / len(v) * 1e-3) / 1e9, 1)}
                        for k, v in summ.items()}}, warm + reps


def figures(times, name, n, workers):
    avg_ms = sum(times) / len(times)
    bpe = kernel_bytes_per_elem(name, workers)
    gbs = bpe * n / (avg_ms * 1e-3) / 1e9
    return {"calls": len(times), "avg_ms": round(avg_ms, 4),
            "median_ms": round(sorted(times)[len(times) // 2], 4), "min_ms": round(min(times), 4),
            "bytes_per_elem": bpe, "GB/s": round(gbs, 1),
            "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4), "elements/s": n / (avg_ms * 1e-3)}


def profiled_traffic(workload, kernel):
    """HBM bytes per element of `kernel` as rocprofv3's FETCH_SIZE / WRITE_SIZE counters gave
    them for this workload: read from the committed summary of those two counter runs (written
    by --summarize-rocprof), not measured by this run."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_B_PER_ELEM_JSON "):
                table = json.loads(line.split(" ", 1)[1])
                return table.get(kernel), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def main():
    args = parse()
    if args.summarize_rocprof is not None:
        return summarize_rocprof(args.summarize_rocprof)
    if args.gpus != 1:
        print("bench.py: this path is measured on ONE GPU; --gpus above 1 is not supported "
              "(no collectives are part of this build).", file=sys.stderr)
        return 2

    import torch
    import paper_2406_02613_amd as A
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    A.binding.lib()
    w = synth.WORKLOADS[args.workload]
    h = w.hyper
    if args.two_stream:
        return bench_two_stream(args, torch, A, w)
    if args.scheme is not None:
        return bench_scheme(args, torch, A, w, synth)
    blocked = not args.planar_state and not args.unfused_cast
    stash = not (args.no_bf16_stash or args.base_path)
    main_opts = dict(fused_bf16_out=not args.unfused_cast,
                     fused_publish=not (args.unfused_publish or args.base_path),
                     fused_reduce=not (args.unfused_reduce or args.base_path),
                     bf16_stash=stash and not args.bf16_accumulate, adopt_first=False)
    batched = not args.per_worker_launches
    main_opts["interleaved_comm"] = args.interleaved_comm and not (args.bf16_accumulate
                                                                   or args.base_path)
    n_grad_bufs = sum(w.microbatches(0, k) for k in range(w.workers))

    def make_arena():
        """One allocation for every buffer of the round, large enough to span the memory
        classes; None when the device has too little free memory for it, or when the timings
        the classification rests on are too erratic to trust (e.g. under a counter-collecting
        profiler): then the buffers are plain allocations."""
        need = w.n * (16 + 4 + w.workers * (2 + 2 + 4) + 2 * n_grad_bufs)
        free = torch.cuda.mem_get_info()[0]
        size = min(int(0.82 * free), max(int(2.2 * need), 100 << 30))
        if size < 1.25 * need + (8 << 30):
            return None
        try:
            made = A.HbmArena(size)
        except (A.AccoError, MemoryError, RuntimeError) as e:
            print(f"bench.py: no arena ({e}); plain allocations", file=sys.stderr)
            return None
        if made.n_classes > 4 or len(made.runs) > 16:
            print(f"bench.py: memory classes not measurable here ({made.n_classes} classes in "
                  f"{len(made.runs)} runs); plain allocations", file=sys.stderr)
            return None
        return made

    def build(arena):
        owner = A.ShardOwner(w.n, w.workers, A.make_hyper(h.lr, h.beta1, h.beta2, h.eps,
                                                          h.weight_decay),
                             arena=arena, gradient_buffers=n_grad_bufs,
                             blocked_state=blocked, block_elems=args.block_elems,
                             bf16_stash=not args.bf16_accumulate,        # allocate the stash buffers
                             bf16_accumulate=args.bf16_accumulate, batched=batched,
                             interleaved_comm=main_opts["interleaved_comm"],
                             comm_block_elems=args.comm_block_elems)
        owner.set_options(**main_opts)
        scratch = (owner.acc if owner.acc else
                   [torch.empty(w.n, dtype=torch.float32, device="cuda") for _ in range(2)])
        w.device_theta(scratch[0])                        # a planar scratch the round overwrites
        owner.set_state("theta", scratch[0])
        grads, n_bufs = make_grads(torch, synth, w, owner)
        return owner, scratch, grads, n_bufs

    arena = None if args.no_arena else make_arena()
    try:
        owner, scratch, grads, n_bufs = build(arena)
    except MemoryError as e:
        if arena is None:
            raise
        print(f"bench.py: the arena cannot hold the round ({e}); plain allocations",
              file=sys.stderr)
        arena = None
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        owner, scratch, grads, n_bufs = build(None)

    if args.calibrate_copy:
        scratch[1].copy_(scratch[0])           # planar fp32: 4n bytes read, 4n bytes written
        torch.cuda.synchronize()

    log = EventLog(torch)
    owner.trace = log
    for r in range(args.warmup):
        run_round(owner, w, grads)
    torch.cuda.synchronize()

    log.enabled = True
    t_start = torch.cuda.Event(enable_timing=True)
    t_end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    t_start.record()
    for r in range(args.steps):
        run_round(owner, w, grads)
    t_end.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    owner.trace = None
    ms_per_step = t_start.elapsed_time(t_end) / args.steps

    # the same rounds once more without the per-kernel event pairs: what the instrumentation
    # costs (nothing at 875M elements; a third of the round on the cache-resident tiny workload)
    u0, u1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    u0.record()
    for r in range(args.steps):
        run_round(owner, w, grads)
    u1.record()
    torch.cuda.synchronize()
    plain_ms_per_step = u0.elapsed_time(u1) / args.steps

    # ---- outside the timed region: is the state the timed rounds left the right one?
    checks = []
    replay = None
    if not args.no_check:
        replay = OracleReplay(w, "bf16" if args.bf16_accumulate else "f32")
        snap = replay.snapshot(torch, owner)
        replay.run(args.warmup + 2 * args.steps)
        checks.append(dict(replay.compare(snap), after="timed rounds"))

    # The same round on the five base entry points only (acco_accumulate, acco_cast_params as the
    # publish, acco_reduce_shards, acco_estimate_step, acco_commit_step with its bf16 output), on
    # the same buffers and continuing from the same state: what the fusions and the stash are worth.
    base_round = adopted_round = None
    extras = not args.no_extras and not args.bf16_accumulate
    if extras and not args.base_path:
        owner.set_options(fused_publish=False, fused_reduce=False, bf16_stash=False,
                          interleaved_comm=False)
        owner.batched = False
        base_round, done = time_rounds(torch, owner, w, grads, max(2, min(5, args.steps)))
        if replay is not None:
            snap = replay.snapshot(torch, owner)
            replay.run(done)
            checks.append(dict(replay.compare(snap), after="base-entry-point rounds"))
        owner.batched = batched
    # The default path once more with the first micro-batch of every accumulation used in place
    # as the stash (no acco_accumulate_first copy): valid for a caller whose backward pass writes
    # that gradient into a buffer it then leaves alone, as the resident gradients here are.
    if extras and main_opts["bf16_stash"] and main_opts["fused_publish"]:
        owner.set_options(**dict(main_opts, adopt_first=True))
        adopted_round, done = time_rounds(torch, owner, w, grads, max(2, min(5, args.steps)))
        if replay is not None:
            snap = replay.snapshot(torch, owner)
            replay.run(done)
            checks.append(dict(replay.compare(snap), after="adopted-first-gradient rounds"))
    # The default path once more with the whole round recorded as one HIP graph: the step
    # kernels read their scalars from a device block that is refilled before every replay, so
    # the update index moves on; from the host a round is two launches (the scalars, the graph).
    recorded_round = None
    if extras and not args.base_path:
        owner.set_options(**dict(main_opts, device_scalars=True))
        run_round(owner, w, grads)          # eagerly once: every *_dev kernel has run before the capture
        rec = owner.record_round(grads[synth.STAGE_TILDE], grads[synth.STAGE_FULL])
        rec.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        host0 = time.perf_counter()
        g0.record()
        for r in range(args.steps):
            rec.replay()
        g1.record()
        host_ms = (time.perf_counter() - host0) * 1e3 / args.steps
        torch.cuda.synchronize()
        rec_ms = g0.elapsed_time(g1) / args.steps
        recorded_round = {"ms_per_step": round(rec_ms, 4), "steps": args.steps,
                          "elements/s": w.n / (rec_ms * 1e-3),
                          "host_launches_per_step": 2,
                          "host_enqueue_ms_per_step": round(host_ms, 4)}
        if replay is not None:
            snap = replay.snapshot(torch, owner)
            replay.run(2 + args.steps)
            checks.append(dict(replay.compare(snap), after="recorded-graph rounds"))
        del rec
    owner.set_options(**dict(main_opts, device_scalars=False))
    replay = None

    # ---- acco_commit_step and acco_estimate_step on their own (gsum already reduced): the
    # kernels the bandwidth target is stated on.  Same buffers; for the 875M-element workloads
    # at both headline shard lengths (the interleaved state buffer has room for the 37 more).
    B = A.binding
    sizes = [w.n]
    if w.n in HEADLINE_SIZES and blocked:
        sizes = list(HEADLINE_SIZES)
    try:
        out_bf16 = (torch.empty(max(sizes), dtype=torch.bfloat16, device="cuda") if arena is None
                    else arena.alloc(max(sizes), torch.bfloat16, owner.roles["out"]))
    except MemoryError:
        out_bf16 = torch.empty(max(sizes), dtype=torch.bfloat16, device="cuda")
    standalone = {}
    for n_k in sizes:
        solo = EventLog(torch)
        solo.enabled = True
        o16 = out_bf16[:n_k]
        cnt = max(owner.total.value, 1)
        for _ in range(max(3, args.steps) + 1):
            solo("commit_bf16", B.acco_commit_step, owner.theta, owner.m, owner.v, owner.gsum,
                 owner.hp, owner.step, cnt, theta_bf16=o16, n=n_k)
            solo("commit", B.acco_commit_step, owner.theta, owner.m, owner.v, owner.gsum,
                 owner.hp, owner.step, cnt, n=n_k)
            solo("estimate", B.acco_estimate_step, owner.theta, owner.m, owner.v, owner.gsum,
                 owner.hp, owner.step.value, cnt, theta_tilde_bf16=o16, n=n_k)
        torch.cuda.synchronize()
        standalone[str(n_k)] = {name: figures(ts[1:], name, n_k, w.workers)
                                for name, ts in solo.summary().items()}
    del out_bf16

    # What the memory system gives for the same access patterns without the arithmetic
    # (planar fp32 arrays borrowed from the accumulators): context for the figures above.
    ceilings = {}
    if extras and len(owner.acc) >= 4:
        probe = EventLog(torch)
        probe.enabled = True
        a4 = owner.acc[:4]
        for _ in range(6):
            probe("copy", B.acco_probe_copy, a4[0], a4[1])
            probe("triad", B.acco_probe_triad, a4[0], a4[1], a4[2], a4[3])
            probe("memcpy", a4[2].copy_, a4[3])
        torch.cuda.synchronize()
        for name, bpe, label in (("copy", 8, "device_copy_kernel"), ("memcpy", 8, "hipMemcpy_d2d"),
                                 ("triad", 28, "triad_4_reads_3_writes_in_place")):
            ts = probe.summary().get(name, [])[1:]
            if ts:
                ms = sum(ts) / len(ts)
                ceilings[label] = {"avg_ms": round(ms, 4), "bytes_per_elem": bpe,
                                   "GB/s": round(bpe * w.n / (ms * 1e-3) / 1e9, 1)}

    kernels = {}
    for name, times in log.summary().items():
        kernels[name] = dict(figures(times, name, w.n, w.workers),
                             calls_per_step=len(times) / args.steps)
        del kernels[name]["calls"]
    bytes_per_round = sum(k["bytes_per_elem"] * k["calls_per_step"] for k in kernels.values())

    # roofline: the committed step with its fused bf16 output on its own, at the workload's
    # length; next to it the other headline length and the committed-step kernel of the round
    head = standalone[str(w.n)]["commit_bf16"]
    traffic, traffic_src = profiled_traffic(w.name, "commit_bf16")
    round_head = next((k for k in ("reduce_commit_bf16", "reduce_commit", "commit_bf16", "commit")
                       if k in kernels), None)
    roofline = {"kernel": "acco_commit_step (fused bf16 output), on its own after the timed region",
                "bound": "hbm", "achieved": head["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": head["frac_of_peak"], "n": w.n,
                "bytes_per_launch": head["bytes_per_elem"] * w.n, "avg_ms": head["avg_ms"],
                # counters of an earlier rocprofv3 run of this command, kept under profiles/
                "traffic": None if traffic is None else traffic * w.n,
                "traffic_source": traffic_src,
                "headline_sizes": {n_k: {name: {"GB/s": f["GB/s"], "frac": f["frac_of_peak"],
                                                "avg_ms": f["avg_ms"],
                                                "bytes_per_elem": f["bytes_per_elem"]}
                                         for name, f in tab.items()}
                                   for n_k, tab in standalone.items()}}
    if round_head is not None:
        k = kernels[round_head]
        rt, _ = profiled_traffic(w.name, round_head)
        roofline["in_timed_round"] = {
            "kernel": {"reduce_commit_bf16": "acco_reduce_commit_step (fused bf16 output)",
                       "reduce_commit": "acco_reduce_commit_step",
                       "commit_bf16": "acco_commit_step (fused bf16 output)",
                       "commit": "acco_commit_step"}[round_head],
            "achieved": k["GB/s"], "frac": k["frac_of_peak"], "avg_ms": k["avg_ms"],
            "bytes_per_launch": k["bytes_per_elem"] * w.n,
            "traffic": None if rt is None else rt * w.n}

    ok = all(c["ok"] for c in checks)
    out = {
        "metric": "shard optimizer-step elements/s + achieved HBM GB/s vs MI355X peak",
        "metric_detail": "value = shard elements / time of one full ACCO round of one shard owner "
                         "(all micro-batch accumulations, publishes, both reductions, estimate, "
                         "commit); achieved GB/s per kernel in roofline / kernels",
        "value": w.n / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n}-element fp32 shard (theta, m, v), W={w.workers} "
                               f"simulated workers, {sum(w.microbatches(0, k) for k in range(w.workers))} "
                               f"bf16 micro-batch gradients per round, AdamW lr={h.lr} "
                               f"betas=({h.beta1},{h.beta2}) eps={h.eps} wd={h.weight_decay}",
                   "n": w.n, "workers": w.workers,
                   "sequenced_by": "paper_2406_02613_amd.ShardOwner",
                   "resident_gradient_buffers": n_bufs,
                   "state_layout": (f"theta,m,v,gsum interleaved in blocks of {args.block_elems} "
                                    "elements" if blocked else "planar"),
                   "fused_bf16_output": main_opts["fused_bf16_out"],
                   "fused_publish": main_opts["fused_publish"],
                   "bf16_stash_of_first_microbatch": main_opts["bf16_stash"],
                   "accumulator_dtype": "bf16" if args.bf16_accumulate else "f32",
                   "fused_reduce": main_opts["fused_reduce"],
                   "one_accumulate_launch_for_all_workers": batched,
                   "communication_buffers": (f"interleaved in blocks of {args.comm_block_elems} "
                                             "elements" if main_opts["interleaved_comm"]
                                             else "planar, one allocation per worker"),
                   "placement": ("one arena, buffers placed by memory class: " + arena.describe()
                                 + "; classes of the roles: " + json.dumps(owner.roles)
                                 if arena is not None else "plain allocations"),
                   "launches_per_step": sum(k["calls_per_step"] for k in kernels.values()),
                   "bytes_per_elem_per_step": bytes_per_round,
                   "host_wall_ms_per_step": wall * 1e3 / args.steps,
                   "ms_per_step_without_per_kernel_events": plain_ms_per_step},
        "round_GB/s": round(bytes_per_round * w.n / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "kernels": kernels,
        # were the timed rounds (and the extra rounds after them) the right computation?  The
        # state on sampled index ranges against the CPU oracle's binary32 form, bit for bit.
        "checked": bool(checks) and ok,
        "check": checks or "skipped (--no-check)",
        # acco_commit_step / acco_estimate_step launched on their own after the timed region
        # (gsum already reduced), per shard length
        "standalone_step_kernels": standalone,
        # the round again on the five base entry points only (no fused entry point, no stash)
        "base_entry_points_round": base_round,
        # the default path with the first gradient of each accumulation adopted in place (an
        # option for callers that leave that buffer alone; not the headline figure)
        "adopted_first_gradient_round": adopted_round,
        # the default path with each round replayed from one recorded HIP graph (device-resident
        # step scalars); same values, checked like the others
        "recorded_graph_round": recorded_round,
        # plain streaming kernels with the same access patterns and no arithmetic, same buffers
        "memory_system_reference": ceilings,
        # The paper times whole training runs, not this path; its wall-clock table (ZeRO-1 vs
        # ACCO, other hardware) is carried here as context only, never as a target.
        "paper_context": PAPER_CONTEXT,
    }
    if not args.no_cpu_baseline:
        del grads
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds,
                                           "bf16" if args.bf16_accumulate else "f32")
    print(json.dumps(out))
    return 0 if (ok or not checks) else 1


if __name__ == "__main__":
    sys.exit(main())
