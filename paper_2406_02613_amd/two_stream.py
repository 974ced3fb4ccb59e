"""The two streams of Alg. 1 on one GPU (Alg. 1, computation stream / communication stream).

A computation stream keeps accumulating micro-batch gradients on whichever parameter version
it was last handed, while a communication stream runs the shard owner's stage in parallel:
publish, reduce, then the speculative estimate (first stage of a round) or the committed update
(second stage).  The streams meet only at the hand-off: when the owner's stage is done it raises
a ready flag; the computation stream, on seeing it, takes the new parameters, gives up what it
has accumulated so far together with its count, and starts the next accumulation.  How many
micro-batches a stage accumulates is therefore decided at run time by how long the other stream
takes - the method's "accumulate while you communicate".

This GPU plays worker 0 and the owner of the shard; the other W-1 workers are represented by
their published bf16 buffers and counts, which the caller provides.  The ready flags are HIP
events on the communication stream that the host polls after each micro-batch.

Host-side sequencing only; all arithmetic is in the C-ABI library.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

from . import binding as B
from .state import BlockedState


@dataclass
class StageRecord:
    round: int
    stage: int                 # 1 or 2
    microbatches: int          # accumulated by worker 0 while the other stream worked
    total_count: int           # micro-batches in the reduced gradient used by this stage's Opt
    comm_ms: float = 0.0       # duration of the stage on the communication stream
    comp_ms: float = 0.0       # duration of the accumulation loop on the computation stream


@dataclass
class TwoStreamLog:
    stages: List[StageRecord] = field(default_factory=list)

    def extra_accumulations(self, minimum: int = 1) -> int:
        """Micro-batches beyond the minimum per stage: the 'supplementary accumulation steps'
        the paper's scheduler adds while communication is in flight."""
        return sum(max(0, s.microbatches - minimum) for s in self.stages)


class TwoStreamOwner:
    def __init__(self, n: int, workers: int, hp: B.AdamW, *, blocked_state: bool = True,
                 device="cuda", arena=None):
        """arena: an arena.HbmArena to place the buffers by memory class (what the owner's
        kernels read together in one class, what the accumulation reads together in another,
        the parameter output in a third); the peers' buffers and the gradients then come from
        ``new_buffer``."""
        import torch
        self.torch = torch
        self.n, self.W, self.hp = int(n), int(workers), hp
        f32, bf16 = torch.float32, torch.bfloat16
        dev = torch.device(device)
        self._dev, self.arena = dev, arena
        self.roles = {}              # with an arena: memory class of each role's buffers
        if arena is not None:
            from .arena import plan_roles
            self.roles = plan_roles(arena, {"owner": 16 * self.n + 2 * self.n * self.W,
                                             "compute": 14 * self.n})
        if blocked_state:
            self.state = BlockedState(n, device=dev, alloc=None if arena is None else (
                lambda numel, dt: self.new_buffer("owner", numel, dt, zero=True)))
            self.theta, self.m, self.v, self.gsum = (self.state.theta, self.state.m,
                                                     self.state.v, self.state.gsum)
        else:
            self.state = None
            self.theta = self.new_buffer("owner", n, f32)
            self.m = self.new_buffer("owner", n, f32, zero=True)
            self.v = self.new_buffer("owner", n, f32, zero=True)
            self.gsum = self.new_buffer("owner", n, f32)
        # worker 0: the two gradient accumulators of Alg. 1 (g and g~) and its comm buffer
        self.acc = {1: self.new_buffer("compute", n, f32),         # g~ (consumed by stage 1)
                    2: self.new_buffer("compute", n, f32)}         # g  (consumed by stage 2)
        self.count = {1: B.Counter(0), 2: B.Counter(0)}
        # the first micro-batch of each accumulation is kept as bf16 (exact), see binding
        self.stash = {1: self.new_buffer("compute", n, bf16),
                      2: self.new_buffer("compute", n, bf16)}
        self.comm0 = self.new_buffer("owner", n, bf16)
        self.params_bf16 = self.new_buffer("out", n, bf16)   # Buffer_i as the compute side sees it
        self.total = B.Counter(0)
        self.step = B.Counter(0)
        self.comp_stream = torch.cuda.Stream()
        self.comm_stream = torch.cuda.Stream()

    def new_buffer(self, role: str, numel: int, dtype, zero: bool = False):
        """A flat buffer for `role`: "owner" (read by the owner's stage: state, published
        buffers of all workers), "compute" (read by the accumulation: accumulators, stashes,
        micro-batch gradients) or "out"; from the arena in that role's class if there is one."""
        if self.arena is None:
            make = self.torch.zeros if zero else self.torch.empty
            return make(int(numel), dtype=dtype, device=self._dev)
        return self.arena.alloc(numel, dtype, self.roles[role], zero=zero)

    def new_peer_buffer(self, worker: int):
        """The published bf16 buffer of another worker (1 .. W-1), placed with the owner's
        buffers and staggered by 4 KiB per worker like shard.ShardOwner's."""
        from .shard import COMM_SKEW_BYTES
        skew = (worker % 8) * (COMM_SKEW_BYTES // 2)
        return self.new_buffer("owner", self.n + skew, self.torch.bfloat16)[skew:skew + self.n]

    def set_theta(self, planar) -> None:
        if self.state is not None:
            self.state.load("theta", planar)
        else:
            self.theta.copy_(planar)

    def get_state(self, name: str):
        return self.state.planar(name) if self.state is not None else getattr(self, name)

    # ------------------------------------------------------------------ one stage of each stream
    def _communicate(self, stage: int, peers: Sequence, peer_counts: Sequence[int],
                     transport: Optional[Callable[[], None]] = None):
        """Enqueue the owner's stage on the communication stream; returns (start, done) events.
        `transport`, if given, is enqueued where the Reduce_Scatter's transfer would sit (between
        the publish and the owner-side reduction), e.g. a timed wait standing in for the links."""
        torch = self.torch
        with torch.cuda.stream(self.comm_stream):
            start = torch.cuda.Event(enable_timing=True)
            done = torch.cuda.Event(enable_timing=True)
            start.record()
            if self.count[stage].value == 1:                          # Buffer_i <- (N, g)
                B.acco_accumulate_first(self.comm0, self.stash[stage], True)
            else:
                B.acco_cast_params(self.comm0, self.acc[stage])
            if transport is not None:
                transport()
            shards = [self.comm0, *peers]
            counts = [self.count[stage].value, *peer_counts]
            if stage == 1:
                B.acco_reduce_estimate_step(self.theta, self.m, self.v, self.gsum, shards, counts,
                                            self.total, self.hp, self.step.value,
                                            theta_tilde_bf16=self.params_bf16, n=self.n)
            else:
                B.acco_reduce_commit_step(self.theta, self.m, self.v, self.gsum, shards, counts,
                                          self.total, self.hp, self.step,
                                          theta_bf16=self.params_bf16, n=self.n)
            done.record()
        return start, done

    def _accumulate_until(self, stage: int, ready, next_grad: Callable[[int], object],
                          compute: Optional[Callable[[], None]], max_microbatches: int,
                          min_microbatches: int = 1):
        """Computation stream: micro-batches into acc[stage] until `ready` has fired (at least
        min_microbatches, at most max_microbatches).  Returns (count, start event, end event)."""
        torch = self.torch
        k = 0
        with torch.cuda.stream(self.comp_stream):
            start = torch.cuda.Event(enable_timing=True)
            start.record()
            while True:
                if compute is not None:
                    compute()                                         # forward/backward stand-in
                g = next_grad(k)                                      # bf16 gradient of micro-batch k
                if k == 0:
                    B.acco_accumulate_first(self.stash[stage], g, False, self.count[stage])
                elif k == 1:
                    B.acco_accumulate_second(self.stash[stage], g, acc=self.acc[stage],
                                             count=self.count[stage])
                else:
                    B.acco_accumulate(self.acc[stage], g, False, self.count[stage])
                k += 1
                mark = torch.cuda.Event()
                mark.record()
                mark.synchronize()                # the loop test happens after the micro-batch
                if k >= max_microbatches:
                    break
                if k >= min_microbatches and (ready is None or ready.query()):
                    break
            end = torch.cuda.Event(enable_timing=True)
            end.record()
        return k, start, end

    # ------------------------------------------------------------------ the training loop
    def run(self, rounds: int, grad_source: Callable[[int, int, int], object],
            peers: Sequence, peer_counts: Sequence[int],
            compute: Optional[Callable[[], None]] = None,
            max_microbatches: int = 64,
            min_microbatches: Callable[[int, int], int] = lambda rnd, acc: 1,
            transport: Optional[Callable[[], None]] = None) -> TwoStreamLog:
        """`grad_source(round, acc, k)` returns worker 0's k-th bf16 micro-batch gradient
        accumulated during round `round` into accumulator `acc` (1: g~, consumed by stage 1 of
        the NEXT round; 2: g, consumed by stage 2 of the same round); round -1 is the
        initialisation gradient.  The tensor must be valid on the computation stream.
        `peers`: W-1 published bf16 buffers, reused every stage, with `peer_counts`.
        `min_microbatches(round, acc)`: the planned accumulation steps; more are added while
        the communication stream is still busy."""
        torch = self.torch
        assert len(peers) == self.W - 1 == len(peer_counts)
        log = TwoStreamLog()
        torch.cuda.synchronize()
        # Initialisation line of Alg. 1: one gradient for g~ before anything is communicated.
        k, _, _ = self._accumulate_until(1, None, lambda j: grad_source(-1, 1, j), compute, 1)
        self.comp_stream.synchronize()
        pending = []
        for t in range(rounds):
            for stage in (1, 2):
                # hand the finished accumulator to the communication stream ...
                self.comm_stream.wait_stream(self.comp_stream)
                c_start, c_done = self._communicate(stage, peers, peer_counts, transport)
                # ... and keep accumulating the other one until that stage reports ready
                other = 2 if stage == 1 else 1
                kk, a_start, a_end = self._accumulate_until(
                    other, c_done, lambda j, r=t, s=other: grad_source(r, s, j), compute,
                    max_microbatches, max(1, int(min_microbatches(t, other))))
                self.comm_stream.synchronize()
                rec = StageRecord(t, stage, kk, self.total.value)
                pending.append((rec, c_start, c_done, a_start, a_end))
                log.stages.append(rec)
        torch.cuda.synchronize()
        for rec, cs, cd, a_s, a_e in pending:
            rec.comm_ms = cs.elapsed_time(cd)
            rec.comp_ms = a_s.elapsed_time(a_e)
        return log
