"""Update schemes of the paper's Sec. 3.1-3.2 sequenced on one shard owner's kernels.

  ddp   eq. (DDP):  theta(t+1) = Opt(theta(t), g(t));                 compute waits for it
  dpu   eq. (DPU):  theta(t+1) = Opt(theta(t), g(t)),  theta~(t+1) = theta(t)
  wp    eq. (WP):   theta(t+1) = Opt(theta(t), g(t)),  theta~(t+1) = Opt(theta(t+1), g(t))
  acco  eq. (ACCO): theta~(t+1) = Opt(theta(t), g~(t)),
                    theta(t+1)  = Opt(theta(t), (g(t) + g~(t)) / 2)

with Opt = AdamW or plain SGD (the optimizer of the convergence propositions).  Host-side
ordering of C-ABI calls only; ``params_f32`` / ``params_bf16`` are the parameters the
computation stream differentiates next (theta~ in the paper's notation, or theta for ddp).

``warmup_rounds`` (dpu only): the first rounds run undelayed, as ddp, before the delayed
updates start - the warm-up the paper's experiment on the impact of delayed updates varies
(Sec. 4, none / 40 / 500 steps).
"""
from __future__ import annotations

from typing import List

from . import binding as B

SCHEMES = ("acco", "ddp", "dpu", "wp")


class SchemeOwner:
    def __init__(self, n: int, workers: int, scheme: str, opt, *, comm_bf16: bool = True,
                 device="cuda", warmup_rounds: int = 0, arena=None):
        """arena: an arena.HbmArena to place the buffers by memory class (state and
        communication buffers in one class, accumulators and the gradients from
        ``new_gradient_buffer`` in another, the parameter outputs in a third)."""
        import torch
        if scheme not in SCHEMES:
            raise ValueError(f"scheme must be one of {SCHEMES}")
        if warmup_rounds < 0 or (warmup_rounds and scheme != "dpu"):
            raise ValueError("warmup_rounds: a non-negative number of undelayed rounds, dpu only")
        self.warmup_rounds = int(warmup_rounds)
        self.rounds_done = 0
        if not isinstance(opt, (B.AdamW, B.Sgd)):
            raise TypeError("opt: an AdamW or Sgd hyper-parameter struct")
        self.torch, self.scheme, self.opt = torch, scheme, opt
        self.adam = isinstance(opt, B.AdamW)
        self.n, self.W, self.comm_bf16 = int(n), int(workers), comm_bf16
        f32, bf16 = torch.float32, torch.bfloat16
        self._dev, self.arena, self.roles = torch.device(device), arena, {}
        if arena is not None:
            from .arena import plan_roles
            self.roles = plan_roles(arena, {
                "owner": 16 * self.n + (2 * self.n * self.W if comm_bf16 else 0),
                "compute": 4 * self.n * self.W + 2 * self.n * 4 * self.W})
        self.theta = self._alloc("owner", n, f32)
        self.m = self._alloc("owner", n, f32, zero=True) if self.adam else None
        self.v = self._alloc("owner", n, f32, zero=True) if self.adam else None
        self.gsum = self._alloc("owner", n, f32)
        self.acc: List = [self._alloc("compute", n, f32) for _ in range(workers)]
        # the W buffers staggered by 4 KiB each, as in shard.ShardOwner
        from .shard import COMM_SKEW_BYTES
        skew = COMM_SKEW_BYTES // 2
        self.comm: List = ([self._alloc("owner", n + (w % 8) * skew, bf16)[(w % 8) * skew:
                                                                         (w % 8) * skew + n]
                            for w in range(workers)] if comm_bf16 else [])
        self.params_f32 = self._alloc("out", n, f32)
        self.params_bf16 = self._alloc("out", n, bf16)
        self.count = [B.Counter(0) for _ in range(workers)]
        self.total = B.Counter(0)
        self.step = B.Counter(0)
        self._fresh = [True] * workers

    def _alloc(self, role: str, numel: int, dtype, zero: bool = False):
        if self.arena is None:
            make = self.torch.zeros if zero else self.torch.empty
            return make(int(numel), dtype=dtype, device=self._dev)
        return self.arena.alloc(numel, dtype, self.roles[role], zero=zero)

    def new_gradient_buffer(self):
        """An n-element bf16 buffer for a micro-batch gradient, in the accumulators' class."""
        return self._alloc("compute", self.n, self.torch.bfloat16)

    @property
    def params(self):
        """fp32 parameters the computation stream differentiates next."""
        return self.params_f32

    def set_theta(self, theta) -> None:
        """Initial parameters; the computation stream starts from the same values."""
        self.theta.copy_(theta)
        self._export_theta()

    # ---------------------------------------------------------------- gradients in
    def add_microbatch(self, worker: int, grad_bf16) -> None:
        B.acco_accumulate(self.acc[worker], grad_bf16, self._fresh[worker], self.count[worker])
        self._fresh[worker] = False

    def set_gradient_f32(self, worker: int, grad_f32, count: int = 1) -> None:
        """Hand over a worker's already accumulated fp32 gradient (fp32 communication only)."""
        if self.comm_bf16:
            raise ValueError("set_gradient_f32 needs comm_bf16=False")
        self.acc[worker].copy_(grad_f32)
        self.count[worker].value = int(count)
        self._fresh[worker] = False

    # ---------------------------------------------------------------- building blocks
    def _reduce(self, accumulate: bool) -> None:
        shards = self.acc
        if self.comm_bf16:
            for w in range(self.W):
                B.acco_cast_params(self.comm[w], self.acc[w])
            shards = self.comm
        B.acco_reduce_shards(self.gsum, shards, accumulate, [c.value for c in self.count],
                             self.total)
        self._fresh = [True] * self.W

    def _estimate(self) -> None:
        if self.adam:
            B.acco_estimate_step(self.theta, self.m, self.v, self.gsum, self.opt, self.step.value,
                                 self.total.value, theta_tilde_f32=self.params_f32,
                                 theta_tilde_bf16=self.params_bf16)
        else:
            B.acco_sgd_estimate_step(self.theta, self.gsum, self.opt, self.total.value,
                                     theta_tilde_f32=self.params_f32,
                                     theta_tilde_bf16=self.params_bf16)

    def _commit(self) -> None:
        if self.adam:
            B.acco_commit_step(self.theta, self.m, self.v, self.gsum, self.opt, self.step,
                               self.total.value)
        else:
            B.acco_sgd_commit_step(self.theta, self.gsum, self.opt, self.step, self.total.value)

    def _export_theta(self) -> None:
        self.params_f32.copy_(self.theta)                 # device copy: plumbing
        B.acco_cast_params(self.params_bf16, self.theta)

    # ---------------------------------------------------------------- the schemes
    def finish_half(self) -> None:
        """ACCO stage (1): the first half's gradients are in; speculate theta~(t+1)."""
        if self.scheme != "acco":
            raise ValueError("only acco has a half-round stage")
        self._reduce(False)
        self._estimate()

    def finish_round(self) -> None:
        if self.scheme == "acco":
            self._reduce(True)                            # onto the retained first-half sum
            self._commit()
            self._export_theta()
        elif self.scheme == "ddp" or self.rounds_done < self.warmup_rounds:
            self._reduce(False)
            self._commit()
            self._export_theta()
        elif self.scheme == "dpu":
            self._export_theta()                          # theta~(t+1) = theta(t)
            self._reduce(False)
            self._commit()
        else:                                             # wp
            self._reduce(False)
            self._commit()
            self._estimate()                              # second Opt step on the same gradient
        self.rounds_done += 1
