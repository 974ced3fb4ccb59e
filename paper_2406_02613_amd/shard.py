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
                 (acco_reduce_estimate_step / acco_reduce_commit_step).
"""
from __future__ import annotations

from typing import List

from . import binding as B


class ShardOwner:
    def __init__(self, n: int, workers: int, hp: B.AdamW, *, device="cuda", comm_bf16: bool = True,
                 fused_bf16_out: bool = True, fused_publish: bool = False,
                 fused_reduce: bool = False, blocked_state: bool = False,
                 block_elems: int = 8192, bf16_stash: bool = False,
                 bf16_accumulate: bool = False, lr_schedule=None, adopt_first: bool = False):
        import torch
        self.torch = torch
        self.n, self.W, self.hp = int(n), int(workers), hp
        # optional: lr_schedule(step) -> learning rate of update number `step` (0-based), e.g.
        # lambda t: acco_lr_cosine(6e-4, 0.0, t, 0, 50000); both stages of a round use the
        # rate of the update they estimate / commit
        self.lr_schedule = lr_schedule
        self.comm_bf16 = comm_bf16
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
        if blocked_state:
            # theta, m, v, gsum interleaved block by block in one buffer (see state.py)
            from .state import BlockedState
            self.state = BlockedState(n, block_elems, dev)
            self.theta, self.m, self.v, self.gsum = (self.state.theta, self.state.m,
                                                     self.state.v, self.state.gsum)
        else:
            self.theta = torch.empty(n, dtype=f32, device=dev)
            self.m = torch.zeros(n, dtype=f32, device=dev)
            self.v = torch.zeros(n, dtype=f32, device=dev)
            self.gsum = torch.empty(n, dtype=f32, device=dev)
        self.acc: List = ([] if bf16_accumulate else
                          [torch.empty(n, dtype=f32, device=dev) for _ in range(workers)])
        self.comm: List = ([torch.empty(n, dtype=bf16, device=dev) for _ in range(workers)]
                           if comm_bf16 else [])
        self.stash: List = ([torch.empty(n, dtype=bf16, device=dev) for _ in range(workers)]
                            if self.bf16_stash and not self.adopt_first else [None] * workers)
        self.theta_tilde_bf16 = torch.empty(n, dtype=bf16, device=dev)
        self.theta_bf16 = torch.empty(n, dtype=bf16, device=dev)
        self.count = [B.Counter(0) for _ in range(workers)]   # N_i of the running accumulation
        self.total = B.Counter(0)                             # micro-batches summed in gsum
        self.step = B.Counter(0)                              # committed updates
        self._fresh = [True] * workers                        # next accumulate starts a new sum
        self._published = [False] * workers                   # comm[w] already written this stage
        self._stashed = [False] * workers                     # the sum so far sits in stash[w]

    # planar access to the state, whatever its layout
    def set_state(self, name: str, planar) -> None:
        if self.state is not None:
            self.state.load(name, planar)
        else:
            getattr(self, name).copy_(planar)

    def get_state(self, name: str):
        return self.state.planar(name) if self.state is not None else getattr(self, name)

    # computation stream
    def add_microbatch(self, worker: int, grad_bf16, last: bool = False) -> None:
        """Accumulate one micro-batch gradient.  ``last`` marks the final micro-batch of the
        stage for this worker (used only with fused_publish)."""
        publish = last and self.fused_publish
        if self.bf16_accumulate:
            B.acco_accumulate_bf16(self.comm[worker], grad_bf16, self._fresh[worker],
                                   self.count[worker])
            self._published[worker] = True
        elif self.adopt_first and self._fresh[worker] and not publish:
            # first micro-batch, used where it lies: no device work, only the bookkeeping
            if grad_bf16.numel() != self.n or grad_bf16.dtype != self.torch.bfloat16:
                raise ValueError("grad_bf16: wrong size or dtype")
            self.stash[worker] = grad_bf16
            self.count[worker].value = 1
            self._stashed[worker] = True
        elif self.bf16_stash and self._fresh[worker]:
            # first micro-batch: kept as bf16; if it is also the last, it IS the published sum
            B.acco_accumulate_first(self.comm[worker] if publish else self.stash[worker],
                                    grad_bf16, publish, self.count[worker])
            self._published[worker] = publish
            self._stashed[worker] = not publish
        elif self.bf16_stash and self._stashed[worker]:
            # second micro-batch: stash + grad in fp32, to the accumulator or straight out
            if (self.adopt_first and self.n > 0
                    and grad_bf16.data_ptr() == self.stash[worker].data_ptr()):
                raise ValueError("the buffer adopted as the first micro-batch was reused")
            if publish:
                B.acco_accumulate_second(self.stash[worker], grad_bf16,
                                         comm_bf16=self.comm[worker], count=self.count[worker])
                self._published[worker] = True
            else:
                B.acco_accumulate_second(self.stash[worker], grad_bf16, acc=self.acc[worker],
                                         count=self.count[worker])
            self._stashed[worker] = False
        elif publish:
            B.acco_accumulate_publish(self.acc[worker], grad_bf16, self.comm[worker],
                                      self._fresh[worker], False, self.count[worker])
            self._published[worker] = True
        else:
            B.acco_accumulate(self.acc[worker], grad_bf16, self._fresh[worker],
                              self.count[worker])
        self._fresh[worker] = False

    def _publish(self):
        for w in range(self.W):
            if self._fresh[w]:
                raise ValueError(f"worker {w} has no micro-batch in this stage (Alg. 1 gives every "
                                 "worker at least one gradient per accumulation)")
        if not self.comm_bf16:
            return self.acc
        for w in range(self.W):
            if self._published[w]:
                continue
            if self._stashed[w]:      # one micro-batch only, not marked last: publish the stash
                B.acco_accumulate_first(self.comm[w], self.stash[w], True)
            else:
                B.acco_cast_params(self.comm[w], self.acc[w])
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
    def stage1(self) -> None:
        shards = self._publish()
        if self.fused_reduce:
            B.acco_reduce_estimate_step(self.theta, self.m, self.v, self.gsum, shards,
                                        self._counts(), self.total, self._hp(), self.step.value,
                                        theta_tilde_bf16=self.theta_tilde_bf16, n=self.n)
        else:
            B.acco_reduce_shards(self.gsum, shards, False, self._counts(), self.total, n=self.n)
            B.acco_estimate_step(self.theta, self.m, self.v, self.gsum, self._hp(), self.step.value,
                                 self.total.value, theta_tilde_bf16=self.theta_tilde_bf16,
                                 n=self.n)
        self._end_stage()

    def stage2(self) -> None:
        shards = self._publish()
        out = self.theta_bf16 if self.fused_bf16_out else None
        if self.fused_reduce:
            B.acco_reduce_commit_step(self.theta, self.m, self.v, self.gsum, shards,
                                      self._counts(), self.total, self._hp(), self.step,
                                      theta_bf16=out, n=self.n)
        else:
            B.acco_reduce_shards(self.gsum, shards, True, self._counts(), self.total, n=self.n)
            B.acco_commit_step(self.theta, self.m, self.v, self.gsum, self._hp(), self.step,
                               self.total.value, theta_bf16=out, n=self.n)
        if not self.fused_bf16_out:
            if self.state is not None:
                raise ValueError("the unfused parameter cast needs a planar theta")
            B.acco_cast_params(self.theta_bf16, self.theta)
        self._end_stage()
