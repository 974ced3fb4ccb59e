"""CPU oracle (TEST INFRASTRUCTURE ONLY) of the update schemes of the paper's Sec. 3.1-3.2 as
one shard owner runs them: eq. (DDP), eq. (DPU), eq. (WP), eq. (ACCO), with Opt = AdamW or
plain SGD.  ``params`` is what the computation stream differentiates next (fp32) and
``params_bf16`` its bf16 copy.  ``warmup_rounds``: undelayed (DDP) rounds before DPU's delayed
updates start (the warm-up of the paper's delayed-update experiment, Sec. 4)."""
from __future__ import annotations

from typing import Optional

import numpy as np

import oracle as O


class OracleScheme:
    def __init__(self, theta: np.ndarray, workers: int, scheme: str, *, adamw: Optional[O.Hyper] = None,
                 sgd_lr: float = 0.0, sgd_wd: float = 0.0, comm_dtype: str = "bf16",
                 precision: str = "f64", warmup_rounds: int = 0):
        assert scheme in ("acco", "ddp", "dpu", "wp")
        assert warmup_rounds == 0 or scheme == "dpu"
        self.warmup_rounds, self.rounds_done = warmup_rounds, 0
        n = theta.size
        self.scheme, self.W, self.precision, self.comm_dtype = scheme, workers, precision, comm_dtype
        self.adamw, self.sgd_lr, self.sgd_wd = adamw, sgd_lr, sgd_wd
        self.theta = theta.astype(np.float32, copy=True)
        self.m = np.zeros(n, np.float32)
        self.v = np.zeros(n, np.float32)
        self.gsum = np.zeros(n, np.float32)
        self.acc = [np.zeros(n, np.float32) for _ in range(workers)]
        self.count = [0] * workers
        self.total = 0
        self.step = 0
        self.params = self.theta.copy()
        self.params_bf16 = O.cast(self.theta)

    def add_microbatch(self, worker: int, grad_bf16: np.ndarray) -> None:
        O.accumulate(self.acc[worker], grad_bf16, init=(self.count[worker] == 0))
        self.count[worker] += 1

    def set_gradient_f32(self, worker: int, grad: np.ndarray, count: int = 1) -> None:
        assert self.comm_dtype == "f32"
        self.acc[worker] = grad.astype(np.float32, copy=True)
        self.count[worker] = count

    def _reduce(self, accumulate: bool) -> None:
        shards = [O.cast(a) for a in self.acc] if self.comm_dtype == "bf16" else self.acc
        O.reduce(self.gsum, shards, accumulate_=accumulate)
        self.total = (self.total if accumulate else 0) + sum(self.count)
        self.count = [0] * self.W

    def _estimate(self) -> None:
        if self.adamw is not None:
            self.params, self.params_bf16 = O.estimate(self.theta, self.m, self.v, self.gsum,
                                                       self.adamw, self.step + 1, self.total,
                                                       precision=self.precision)
        else:
            self.params, self.params_bf16 = O.sgd_step(self.theta, self.gsum, self.sgd_lr,
                                                       self.sgd_wd, self.total, commit=False,
                                                       precision=self.precision)

    def _commit(self) -> None:
        if self.adamw is not None:
            O.commit(self.theta, self.m, self.v, self.gsum, self.adamw, self.step + 1, self.total,
                     want_bf16=False, precision=self.precision)
        else:
            O.sgd_step(self.theta, self.gsum, self.sgd_lr, self.sgd_wd, self.total, commit=True,
                       want_bf16=False, precision=self.precision)
        self.step += 1

    def _export_theta(self) -> None:
        self.params = self.theta.copy()
        self.params_bf16 = O.cast(self.theta)

    def finish_half(self) -> None:
        assert self.scheme == "acco"
        self._reduce(False)
        self._estimate()

    def finish_round(self) -> None:
        if self.scheme == "acco":
            self._reduce(True)
            self._commit()
            self._export_theta()
        elif self.scheme == "ddp" or self.rounds_done < self.warmup_rounds:
            self._reduce(False)
            self._commit()
            self._export_theta()
        elif self.scheme == "dpu":
            self._export_theta()
            self._reduce(False)
            self._commit()
        else:
            self._reduce(False)
            self._commit()
            self._estimate()
        self.rounds_done += 1
