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
"""
from __future__ import annotations

from typing import List, Optional

from . import binding as B


class ShardOwner:
    def __init__(self, n: int, workers: int, hp: B.AdamW, *, device="cuda", comm_bf16: bool = True,
                 fused_bf16_out: bool = True):
        import torch
        self.torch = torch
        self.n, self.W, self.hp = int(n), int(workers), hp
        self.comm_bf16 = comm_bf16
        self.fused_bf16_out = fused_bf16_out
        f32, bf16 = torch.float32, torch.bfloat16
        dev = torch.device(device)
        self.theta = torch.empty(n, dtype=f32, device=dev)
        self.m = torch.zeros(n, dtype=f32, device=dev)
        self.v = torch.zeros(n, dtype=f32, device=dev)
        self.gsum = torch.empty(n, dtype=f32, device=dev)
        self.acc: List = [torch.empty(n, dtype=f32, device=dev) for _ in range(workers)]
        self.comm: List = ([torch.empty(n, dtype=bf16, device=dev) for _ in range(workers)]
                           if comm_bf16 else [])
        self.theta_tilde_bf16 = torch.empty(n, dtype=bf16, device=dev)
        self.theta_bf16 = torch.empty(n, dtype=bf16, device=dev)
        self.count = [B.Counter(0) for _ in range(workers)]   # N_i of the running accumulation
        self.total = B.Counter(0)                             # micro-batches summed in gsum
        self.step = B.Counter(0)                              # committed updates
        self._fresh = [True] * workers                        # next accumulate starts a new sum

    # computation stream
    def add_microbatch(self, worker: int, grad_bf16) -> None:
        B.acco_accumulate(self.acc[worker], grad_bf16, self._fresh[worker], self.count[worker])
        self._fresh[worker] = False

    def _publish(self):
        if not self.comm_bf16:
            return self.acc
        for w in range(self.W):
            B.acco_cast_params(self.comm[w], self.acc[w])
        return self.comm

    def _counts(self) -> List[int]:
        return [c.value for c in self.count]

    # communication stream
    def stage1(self) -> None:
        B.acco_reduce_shards(self.gsum, self._publish(), False, self._counts(), self.total)
        B.acco_estimate_step(self.theta, self.m, self.v, self.gsum, self.hp, self.step.value,
                             self.total.value, theta_tilde_bf16=self.theta_tilde_bf16)
        self._fresh = [True] * self.W

    def stage2(self) -> None:
        B.acco_reduce_shards(self.gsum, self._publish(), True, self._counts(), self.total)
        if self.fused_bf16_out:
            B.acco_commit_step(self.theta, self.m, self.v, self.gsum, self.hp, self.step,
                               self.total.value, theta_bf16=self.theta_bf16)
        else:
            B.acco_commit_step(self.theta, self.m, self.v, self.gsum, self.hp, self.step,
                               self.total.value)
            B.acco_cast_params(self.theta_bf16, self.theta)
        self._fresh = [True] * self.W
