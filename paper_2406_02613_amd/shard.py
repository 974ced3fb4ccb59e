"""One shard owner's buffers in HBM and the call sequence of an ACCO round.

Sequencing only: every arithmetic step, and every counter update, happens inside
the C-ABI library.  The order of calls is the communication stream of Alg. 1 as
the owner of one shard sees it, with the W workers' gradient slices held in this
GPU's memory:

  per micro-batch        acco_accumulate            (g_i += grad, N_i += 1)
  stage 1  publish       acco_cast_params           (Buffer_i <- g~_i, bf16)
           reduce        acco_reduce_shards(init)   (+ sum of the counts)
           estimate      acco_estimate_step         (theta~, nothing committed)
  stage 2  publish       acco_cast_params
           reduce        acco_reduce_shards(accumulate onto the stage-1 sum)
           commit        acco_commit_step           (theta, m, v, step; fused bf16 theta)

Options that give the same values with fewer bytes over HBM:
  bf16_stash     the first micro-batch of an accumulation is kept as bf16 (exact) and the
                 second adds to it in fp32 (acco_accumulate_first / acco_accumulate_second);
  adopt_first    with bf16_stash: the first micro-batch's gradient buffer is used in place as
                 the stash instead of being copied (saves that 4 B/elem pass).  The caller
                 promises not to overwrite that buffer until the worker's next micro-batch has
                 been added or the stage has run - what a framework gets when backward writes
                 its first gradient of an accumulation straight into the accumulation buffer;
  bf16_accumulate  the running sum itself is bf16 and doubles as the communication buffer,
                 the precision of the paper's own setup (acco_accumulate_bf16); this one does
                 change the values: the sum is rounded after every micro-batch;
  fused_publish  the last micro-batch of a stage goes through acco_accumulate_publish,
                 which writes the bf16 communication buffer directly (the caller says which
                 micro-batch is the last one: ``last=True``);
  fused_reduce   reduce + estimate and reduce + commit each run as one kernel
                 (acco_reduce_estimate_step / acco_reduce_commit_step);
  batched        workers that are at the same step of their accumulation share one launch
                 (acco_accumulate_batch) when their gradients are handed over together
                 (add_microbatches / add_microbatch_rows);
  interleaved_comm  the W bf16 communication buffers are the interleaved blocks of one buffer
                 (state.InterleavedShards) instead of W separate ones: same values; the reduce
                 kernels stream them faster and at a speed that does not depend on where W
                 separate buffers happen to lie, the publishing kernels write them slower.
                 Every write to them goes through acco_accumulate_batch, which takes the layout.
  arena          an arena.HbmArena to take every buffer from, placed by memory class: what the
                 step kernels read together (state, communication buffers) in one class, what
                 the accumulation kernels read together (accumulators, stashes, and the
                 gradients the caller gets from ``new_gradient_buffer``) in another, the bf16
                 outputs in a third.  Placement only: same values.
  device_scalars the two AdamW steps read their folded scalars from a small device block that
                 the owner fills before each stage (acco_fold_adamw, acco_stage_scalars, the
                 *_dev step entry points): same values; what it allows is `record_round`, a whole
                 round recorded once as a HIP graph and replayed while the update index moves on.
"""
from __future__ import annotations

from typing import Callable, List, Optional

from . import binding as B

# what ShardOwner.set_options may switch between rounds
COMM_SKEW_BYTES = 4096     # stagger between the workers' planar communication buffers

OPTIONS = ("fused_bf16_out", "fused_publish", "fused_reduce", "bf16_stash", "adopt_first",
           "interleaved_comm", "device_scalars")


class ShardOwner:
    def __init__(self, n: int, workers: int, hp: B.AdamW, *, device="cuda", comm_bf16: bool = True,
                 fused_bf16_out: bool = True, fused_publish: bool = False,
                 fused_reduce: bool = False, blocked_state: bool = False,
                 block_elems: int = 8192, bf16_stash: bool = False,
                 bf16_accumulate: bool = False, lr_schedule=None, adopt_first: bool = False,
                 batched: bool = False, interleaved_comm: bool = False,
                 comm_block_elems: int = 16384, device_scalars: bool = False, arena=None,
                 gradient_buffers: int = 0):
        import torch
        self.torch = torch
        self.n, self.W, self.hp = int(n), int(workers), hp
        # gradient_buffers: how many n-element bf16 gradient buffers the caller will ask
        # new_gradient_buffer for (only used to decide which class gets which role)
        self.arena = arena
        self.roles = {}              # with an arena: memory class of each role's buffers
        if arena is not None:
            from .arena import plan_roles
            n_, W_ = int(n), int(workers)
            self.roles = plan_roles(arena, {
                "owner": 16 * n_ + (2 * n_ * W_ if comm_bf16 else 0),
                "compute": (0 if bf16_accumulate else 4 * n_ * W_) + 2 * n_ * W_
                + 2 * n_ * int(gradient_buffers)})
        # optional: lr_schedule(step) -> learning rate of update number `step` (0-based), e.g.
        # lambda t: acco_lr_cosine(6e-4, 0.0, t, 0, 50000); both stages of a round use the
        # rate of the update they estimate / commit
        self.lr_schedule = lr_schedule
        self.comm_bf16 = comm_bf16
        self.batched = bool(batched)
        self.fused_bf16_out = fused_bf16_out
        self.fused_publish = fused_publish and comm_bf16
        self.fused_reduce = fused_reduce
        self.bf16_accumulate = bf16_accumulate
        if bf16_accumulate and not comm_bf16:
            raise ValueError("bf16 accumulation publishes bf16 buffers")
        self.bf16_stash = bf16_stash and comm_bf16 and not bf16_accumulate
        self.adopt_first = adopt_first and self.bf16_stash
        f32, bf16 = torch.float32, torch.bfloat16
        dev = torch.device(device)
        self.state = None
        self._dev, self._comm_block = dev, int(comm_block_elems)
        if blocked_state:
            # theta, m, v, gsum interleaved block by block in one buffer (see state.py)
            from .state import BlockedState
            self.state = BlockedState(n, block_elems, dev, alloc=None if arena is None else (
                lambda numel, dt: self._alloc("owner", numel, dt, zero=True)))
            self.theta, self.m, self.v, self.gsum = (self.state.theta, self.state.m,
                                                     self.state.v, self.state.gsum)
        else:
            self.theta = self._alloc("owner", n, f32)
            self.m = self._alloc("owner", n, f32, zero=True)
            self.v = self._alloc("owner", n, f32, zero=True)
            self.gsum = self._alloc("owner", n, f32)
        # the communication buffers: W separate ones and / or the interleaved blocks of one
        # buffer, each allocated when first selected
        self._comm_planar: Optional[List] = None
        self._comm_slab = None
        self.interleaved_comm = False
        self.comm: List = []
        self._select_comm(bool(interleaved_comm))
        self._own_stash: List = ([self._alloc("compute", n, bf16) for _ in range(workers)]
                                 if self.bf16_stash and not self.adopt_first else [None] * workers)
        self.stash: List = list(self._own_stash)
        self.acc: List = ([] if bf16_accumulate else
                          [self._alloc("compute", n, f32) for _ in range(workers)])
        self.theta_tilde_bf16 = self._alloc("out", n, bf16)
        self.theta_bf16 = self._alloc("out", n, bf16)
        self.count = [B.Counter(0) for _ in range(workers)]   # N_i of the running accumulation
        self.total = B.Counter(0)                             # micro-batches summed in gsum
        self.step = B.Counter(0)                              # committed updates
        # optional observer of every library call of a round: trace(label, fn, *args, **kw) must
        # return fn(*args, **kw); a benchmark brackets the call with events here, so that what it
        # times is this very sequence and not a copy of it
        self.trace: Optional[Callable] = None
        self._fresh = [True] * workers                        # next accumulate starts a new sum
        self._published = [False] * workers                   # comm[w] already written this stage
        self._stashed = [False] * workers                     # the sum so far sits in stash[w]
        # block 0: the scalars of the estimate, block 1: those of the commit
        self.scalars = None
        self.device_scalars = False
        self._select_scalars(bool(device_scalars))
        self._recording = False

    def _alloc(self, role: str, numel: int, dtype, zero: bool = False):
        """A flat buffer for `role` ("owner", "compute", "out"): from the arena, in that role's
        memory class, or a plain allocation without one."""
        if self.arena is None:
            make = self.torch.zeros if zero else self.torch.empty
            return make(int(numel), dtype=dtype, device=self._dev)
        return self.arena.alloc(numel, dtype, self.roles[role], zero=zero)

    def new_gradient_buffer(self, first: bool = False):
        """An n-element bf16 buffer for a micro-batch gradient, placed where the accumulation
        kernels read it fastest when there is an arena: next to the stashes and accumulators
        it is added to.  ``first``: the buffer will only ever hold the first micro-batch of an
        accumulation; with the bf16 stash that one is merely copied, read together with nothing,
        so it need not take room in that class."""
        if self.bf16_accumulate:
            # the bf16 running sum is the communication buffer itself: the gradients added to
            # it are read together with it; the first one is merely copied
            role = "out" if first else "owner"
        else:
            role = "out" if first and self.bf16_stash and not self.adopt_first else "compute"
        return self._alloc(role, self.n, self.torch.bfloat16)

    def _select_scalars(self, on: bool) -> None:
        if on and self.scalars is None:
            self.scalars = self.torch.zeros(2 * 16, dtype=self.torch.float32, device=self._dev)
        self.device_scalars = on

    def _select_comm(self, interleaved: bool) -> None:
        if not self.comm_bf16:
            self.interleaved_comm, self.comm = False, []
            return
        if interleaved and self.bf16_accumulate:
            raise ValueError("bf16 running sums are updated in place: planar buffers only")
        self.interleaved_comm = interleaved
        if interleaved:
            if self._comm_slab is None:
                from .state import InterleavedShards
                self._comm_slab = InterleavedShards(
                    self.n, self.W, self._comm_block, self._dev,
                    alloc=None if self.arena is None else (
                        lambda numel, dt: self._alloc("owner", numel, dt, zero=True)))
            self.comm = list(self._comm_slab.shards)
        else:
            if self._comm_planar is None:
                # W separate buffers, each started COMM_SKEW_BYTES further into its allocation
                # than the one before: allocations start on 2 MiB boundaries, and W streams read
                # at the same index with identical low address bits queue up on the same DRAM
                # channels (MI355X, W = 8, 875M elements: reduce + estimate 4.46 -> 4.37 ms,
                # reduce + commit 5.98 -> 5.90 with 4 KiB per worker; any multiple of 1 KiB up to
                # 1 MiB helps, 4 and 8 KiB the most)
                skew = COMM_SKEW_BYTES // 2
                self._comm_planar = [
                    self._alloc("owner", self.n + (w % 8) * skew,
                                self.torch.bfloat16)[(w % 8) * skew:(w % 8) * skew + self.n]
                    for w in range(self.W)]
            self.comm = self._comm_planar

    def comm_planar(self, w: int):
        """Worker w's published buffer as a planar tensor of n elements (a copy if interleaved)."""
        return self._comm_slab.planar(w) if self.interleaved_comm else self.comm[w]

    def _call(self, label: str, fn, *args, **kw):
        if self.trace is None:
            return fn(*args, **kw)
        return self.trace(label, fn, *args, **kw)

    def set_options(self, **opts) -> None:
        """Switch fused_bf16_out / fused_publish / fused_reduce / bf16_stash / adopt_first /
        interleaved_comm / device_scalars between rounds (no accumulation may be under way): the values of a round do not depend on them,
        only the calls it is made of.  Buffers are those of the constructor: a stash can only be
        switched on if it was allocated then."""
        if not all(self._fresh):
            raise ValueError("options can only change between stages")
        for k, val in opts.items():
            if k not in OPTIONS:
                raise ValueError(f"unknown option {k!r}")
            if k == "interleaved_comm":
                self._select_comm(bool(val))
            elif k == "device_scalars":
                self._select_scalars(bool(val))
            else:
                setattr(self, k, bool(val))
        self.fused_publish = self.fused_publish and self.comm_bf16
        self.bf16_stash = self.bf16_stash and self.comm_bf16 and not self.bf16_accumulate
        self.adopt_first = self.adopt_first and self.bf16_stash
        if self.bf16_stash and not self.adopt_first and any(t is None for t in self._own_stash):
            raise ValueError("this owner was built without stash buffers")
        self.stash = [None] * self.W if self.adopt_first else list(self._own_stash)
        if not self.fused_bf16_out and self.state is not None:
            raise ValueError("the unfused parameter cast needs a planar theta")

    # planar access to the state, whatever its layout
    def set_state(self, name: str, planar) -> None:
        if self.state is not None:
            self.state.load(name, planar)
        else:
            getattr(self, name).copy_(planar)

    def get_state(self, name: str):
        return self.state.planar(name) if self.state is not None else getattr(self, name)

    # computation stream
    def _step_of(self, worker: int, last: bool) -> str:
        """Which accumulation step the next micro-batch of `worker` is (also its trace label)."""
        publish = last and self.fused_publish
        fresh = self._fresh[worker]
        if self.bf16_accumulate:
            return "accumulate_bf16_init" if fresh else "accumulate_bf16"
        if self.adopt_first and fresh and not publish:
            return "adopt"
        if self.bf16_stash and fresh:
            return "accumulate_first_publish" if publish else "accumulate_first"
        if self.bf16_stash and self._stashed[worker]:
            return "accumulate_second_publish" if publish else "accumulate_second"
        if publish:
            return "accumulate_publish_init" if fresh else "accumulate_publish"
        return "accumulate_init" if fresh else "accumulate"

    # step -> (batched operation, uses acc, output column, uses stash)
    _BATCH = {
        "accumulate_init": (B.BATCH_ACCUMULATE_INIT, True, None, False),
        "accumulate": (B.BATCH_ACCUMULATE, True, None, False),
        "accumulate_publish": (B.BATCH_ACCUMULATE_PUBLISH, True, "comm", False),
        "accumulate_publish_init": (B.BATCH_FIRST_PUBLISH, False, "comm", False),
        "accumulate_first": (B.BATCH_FIRST, False, "stash", False),
        "accumulate_first_publish": (B.BATCH_FIRST_PUBLISH, False, "comm", False),
        "accumulate_second": (B.BATCH_SECOND, True, None, True),
        "accumulate_second_publish": (B.BATCH_SECOND_PUBLISH, False, "comm", True),
        "accumulate_bf16_init": (B.BATCH_FIRST, False, "comm", False),
        "accumulate_bf16": (B.BATCH_RUNNING_BF16, False, "comm", False),
    }

    def _run_step(self, step: str, workers: List[int], grads: List) -> None:
        """Enqueue accumulation step `step` for the listed workers (one gradient each) and do
        the owner's bookkeeping for them."""
        if step == "adopt":
            # first micro-batch, used where it lies: no device work, only the bookkeeping
            for w, g in zip(workers, grads):
                if g.numel() != self.n or g.dtype != self.torch.bfloat16:
                    raise ValueError("grad_bf16: wrong size or dtype")
                self.stash[w] = g
                self.count[w].value = 1
        else:
            if self.adopt_first and step.startswith("accumulate_second") and self.n > 0:
                for w, g in zip(workers, grads):
                    if g.data_ptr() == self.stash[w].data_ptr():
                        raise ValueError("the buffer adopted as the first micro-batch was reused")
            op, use_acc, out, use_stash = self._BATCH[step]
            if (self.batched and len(workers) > 1) or (self.interleaved_comm and out == "comm"):
                cols = {}
                if use_acc:
                    cols["acc"] = [self.acc[w] for w in workers]
                if out is not None:
                    cols["out_bf16"] = [getattr(self, out)[w] for w in workers]
                if use_stash:
                    cols["stash_bf16"] = [self.stash[w] for w in workers]
                self._call(f"{step}*{len(workers)}", B.acco_accumulate_batch, op, self.n,
                           grad_bf16=list(grads), counts=[self.count[w] for w in workers], **cols)
            else:
                for w, g in zip(workers, grads):
                    self._run_single(step, w, g)
        for w in workers:
            if step.startswith("accumulate_bf16") or "publish" in step:
                self._published[w] = True
            self._stashed[w] = step in ("adopt", "accumulate_first")
            self._fresh[w] = False

    def _run_single(self, step: str, w: int, g) -> None:
        cnt = self.count[w]
        if step in ("accumulate_bf16_init", "accumulate_bf16"):
            self._call(step, B.acco_accumulate_bf16, self.comm[w], g, step.endswith("init"), cnt)
        elif step in ("accumulate_first", "accumulate_first_publish"):
            # kept as bf16; if it is also the last micro-batch, it IS the published sum
            publish = step.endswith("publish")
            self._call(step, B.acco_accumulate_first, self.comm[w] if publish else self.stash[w],
                       g, publish, cnt)
        elif step == "accumulate_second_publish":
            self._call(step, B.acco_accumulate_second, self.stash[w], g, comm_bf16=self.comm[w],
                       count=cnt)
        elif step == "accumulate_second":
            self._call(step, B.acco_accumulate_second, self.stash[w], g, acc=self.acc[w], count=cnt)
        elif step in ("accumulate_publish_init", "accumulate_publish"):
            self._call(step, B.acco_accumulate_publish, self.acc[w], g, self.comm[w],
                       step.endswith("init"), False, cnt)
        else:
            self._call(step, B.acco_accumulate, self.acc[w], g, step.endswith("init"), cnt)

    def add_microbatch(self, worker: int, grad_bf16, last: bool = False) -> None:
        """Accumulate one micro-batch gradient.  ``last`` marks the final micro-batch of the
        stage for this worker (used only with fused_publish)."""
        self._run_step(self._step_of(worker, last), [worker], [grad_bf16])

    def add_microbatches(self, items) -> None:
        """Accumulate one micro-batch gradient for each of several workers:
        items = [(worker, grad_bf16, last), ...], every worker at most once.  With
        ``batched`` the workers that are at the same step of their accumulation share one launch."""
        groups = {}
        seen = set()
        for worker, grad, last in items:
            if worker in seen:
                raise ValueError("a worker appears twice in one call")
            seen.add(worker)
            ws, gs = groups.setdefault(self._step_of(worker, last), ([], []))
            ws.append(worker)
            gs.append(grad)
        for step, (ws, gs) in groups.items():
            self._run_step(step, ws, gs)

    def add_microbatch_rows(self, rows) -> None:
        """A whole stage's gradients, rows[worker] = that worker's micro-batch gradients in order
        (the last one of a row is marked as such)."""
        if len(rows) != self.W:
            raise ValueError("one row per worker")
        if self.batched:
            for k in range(max(len(r) for r in rows)):
                self.add_microbatches([(w, r[k], k == len(r) - 1) for w, r in enumerate(rows)
                                       if k < len(r)])
        else:
            for w, r in enumerate(rows):
                for k, g in enumerate(r):
                    self.add_microbatch(w, g, last=(k == len(r) - 1))

    def _publish(self):
        for w in range(self.W):
            if self._fresh[w]:
                raise ValueError(f"worker {w} has no micro-batch in this stage (Alg. 1 gives every "
                                 "worker at least one gradient per accumulation)")
        if not self.comm_bf16:
            return self.acc
        todo = [w for w in range(self.W) if not self._published[w]]
        stashed = [w for w in todo if self._stashed[w]]     # one micro-batch only, not marked last
        summed = [w for w in todo if not self._stashed[w]]
        for ws, label, op, src in ((stashed, "accumulate_first_publish", B.BATCH_FIRST_PUBLISH,
                                    "grad_bf16"), (summed, "cast", B.BATCH_PUBLISH, "acc")):
            if ws and ((self.batched and len(ws) > 1) or self.interleaved_comm):
                col = [self.stash[w] if src == "grad_bf16" else self.acc[w] for w in ws]
                self._call(f"{label}*{len(ws)}", B.acco_accumulate_batch, op, self.n,
                           out_bf16=[self.comm[w] for w in ws], **{src: col})
            elif src == "grad_bf16":
                for w in ws:
                    self._call(label, B.acco_accumulate_first, self.comm[w], self.stash[w], True)
            else:
                for w in ws:
                    self._call(label, B.acco_cast_params, self.comm[w], self.acc[w])
        return self.comm

    def _hp(self) -> B.AdamW:
        if self.lr_schedule is None:
            return self.hp
        h = self.hp
        return B.AdamW(float(self.lr_schedule(self.step.value)), h.beta1, h.beta2, h.eps,
                       h.weight_decay)

    def _counts(self) -> List[int]:
        return [c.value for c in self.count]

    def _end_stage(self) -> None:
        self._fresh = [True] * self.W
        self._published = [False] * self.W
        self._stashed = [False] * self.W
        if self.adopt_first:
            self.stash = [None] * self.W          # the adopted buffers go back to the caller

    # communication stream
    def _stage_scalars(self, block: int, total: int) -> None:
        """Put the scalars of the pending update on `total` micro-batches into scalar block
        `block` (not while a round is being recorded: a replay stages them itself)."""
        if not self._recording:
            self._call("stage_scalars", B.acco_stage_scalars, self.scalars,
                       [B.acco_fold_adamw(self._hp(), self.step.value, total)], block)

    def stage1(self) -> None:
        shards = self._publish()
        if self.device_scalars:
            # the library folds the scalars; the totals are this caller's to keep
            total = sum(self._counts())
            self._stage_scalars(0, total)
            if self.fused_reduce:
                self._call("reduce_estimate", B.acco_reduce_estimate_step_dev, self.theta, self.m,
                           self.v, self.gsum, shards, self.scalars, 0,
                           theta_tilde_bf16=self.theta_tilde_bf16, n=self.n)
            else:
                self._call("reduce_init", B.acco_reduce_shards, self.gsum, shards, False, n=self.n)
                self._call("estimate", B.acco_estimate_step_dev, self.theta, self.m, self.v,
                           self.gsum, self.scalars, 0, theta_tilde_bf16=self.theta_tilde_bf16,
                           n=self.n)
            self.total.value = total
        elif self.fused_reduce:
            self._call("reduce_estimate", B.acco_reduce_estimate_step, self.theta, self.m, self.v,
                       self.gsum, shards, self._counts(), self.total, self._hp(), self.step.value,
                       theta_tilde_bf16=self.theta_tilde_bf16, n=self.n)
        else:
            self._call("reduce_init", B.acco_reduce_shards, self.gsum, shards, False,
                       self._counts(), self.total, n=self.n)
            self._call("estimate", B.acco_estimate_step, self.theta, self.m, self.v, self.gsum,
                       self._hp(), self.step.value, self.total.value,
                       theta_tilde_bf16=self.theta_tilde_bf16, n=self.n)
        self._end_stage()

    def stage2(self) -> None:
        shards = self._publish()
        out = self.theta_bf16 if self.fused_bf16_out else None
        if self.device_scalars:
            total = self.total.value + sum(self._counts())
            self._stage_scalars(1, total)
            if self.fused_reduce:
                self._call("reduce_commit_bf16" if out is not None else "reduce_commit",
                           B.acco_reduce_commit_step_dev, self.theta, self.m, self.v, self.gsum,
                           shards, self.scalars, 1, theta_bf16=out, n=self.n)
            else:
                self._call("reduce_accumulate", B.acco_reduce_shards, self.gsum, shards, True,
                           n=self.n)
                self._call("commit_bf16" if out is not None else "commit", B.acco_commit_step_dev,
                           self.theta, self.m, self.v, self.gsum, self.scalars, 1, theta_bf16=out,
                           n=self.n)
            self.total.value = total
            self.step.value += 1
        elif self.fused_reduce:
            self._call("reduce_commit_bf16" if out is not None else "reduce_commit",
                       B.acco_reduce_commit_step, self.theta, self.m, self.v, self.gsum, shards,
                       self._counts(), self.total, self._hp(), self.step, theta_bf16=out, n=self.n)
        else:
            self._call("reduce_accumulate", B.acco_reduce_shards, self.gsum, shards, True,
                       self._counts(), self.total, n=self.n)
            self._call("commit_bf16" if out is not None else "commit", B.acco_commit_step,
                       self.theta, self.m, self.v, self.gsum, self._hp(), self.step,
                       self.total.value, theta_bf16=out, n=self.n)
        if not self.fused_bf16_out:
            if self.state is not None:
                raise ValueError("the unfused parameter cast needs a planar theta")
            self._call("cast", B.acco_cast_params, self.theta_bf16, self.theta)
        self._end_stage()

    def record_round(self, rows1, rows2) -> "RecordedRound":
        """Record one whole round on fixed gradient buffers as a HIP graph; see RecordedRound."""
        return RecordedRound(self, rows1, rows2)


class RecordedRound:
    """One round of a ShardOwner (both stages of Alg. 1's communication stream with the
    accumulations that feed them) recorded once as a HIP graph.

    rows1[w] / rows2[w]: worker w's micro-batch gradient buffers of the first / second half of
    the round, in order.  The recording keeps their addresses and their number: before each
    `replay` the caller refills the same buffers with the new gradients.  A replay is two
    launches from the host (the scalars of that round's two updates into the owner's device
    block, then the graph) whatever the number of kernels in the round; the update index, the
    learning-rate schedule and the owner's host counters move on as in eager rounds, and the
    values are those of eager rounds bit for bit.

    Recording does no device work and leaves the owner's state and counters as they were.  Every
    kernel of the round should have run once before (an eager round with the same options), so
    that no code object is loaded for the first time inside the capture."""

    def __init__(self, owner: ShardOwner, rows1, rows2):
        torch = owner.torch
        if not owner.device_scalars:
            raise ValueError("record_round needs ShardOwner(device_scalars=True)")
        if not all(owner._fresh):
            raise ValueError("a round can only be recorded between rounds")
        if len(rows1) != owner.W or len(rows2) != owner.W:
            raise ValueError("one row per worker and stage")
        self.owner = owner
        self._rows = ([list(r) for r in rows1], [list(r) for r in rows2])   # keep them alive
        saved = (owner.step.value, owner.total.value, [c.value for c in owner.count], owner.trace)
        owner.trace, owner._recording = None, True
        self.graph = torch.cuda.CUDAGraph()
        try:
            with torch.cuda.graph(self.graph):
                owner.add_microbatch_rows(self._rows[0])
                owner.stage1()
                self.total1 = owner.total.value
                owner.add_microbatch_rows(self._rows[1])
                owner.stage2()
                self.total2 = owner.total.value
            self._end_counts = [c.value for c in owner.count]
            self._totals = (self.total1, self.total2)
            self._stage = B.ScalarStager(owner.scalars, 2)
        finally:
            owner._recording = False
            owner.step.value, owner.total.value, owner.trace = saved[0], saved[1], saved[3]
            for c, x in zip(owner.count, saved[2]):
                c.value = x

    def replay(self) -> None:
        """Enqueue the recorded round on the current stream for the owner's next update."""
        o = self.owner
        if not all(o._fresh):
            raise ValueError("an eager stage is under way")
        step = o.step.value
        self._stage(o._hp(), step, self._totals)
        self.graph.replay()
        for c, x in zip(o.count, self._end_counts):
            c.value = x
        o.total.value = self.total2
        o.step.value = step + 1
