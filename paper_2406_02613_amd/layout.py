"""Buffer inventory of the path: bytes per parameter of each buffer kind.

Follows the paper's mixed-precision setup (Sec. 4.2) and its memory table (Tab. 1):
bf16 parameters, bf16 gradients, a bf16 communication buffer, and K = 12 bytes per
parameter of fp32 optimizer state (theta, m, v) that only the shard owner keeps.
"""
PARAM_BF16 = 2          # model parameters used by forward/backward
GRAD_BF16 = 2           # a micro-batch gradient
COMM_BF16 = 2           # communication buffer (published gradients / gathered parameters)
STATE_F32 = 4 + 4 + 4   # theta, m, v of the sharded optimizer  (K in the paper's table)
ACCUM_F32 = 4           # this implementation's fp32 gradient accumulator (per simulated worker)
GSUM_F32 = 4            # reduced gradient shard


def replica_bytes_per_param(method: str, workers: int) -> float:
    """Per-replica bytes per model parameter as the paper's memory table counts them."""
    if method == "ddp":
        return PARAM_BF16 + GRAD_BF16 + STATE_F32
    if method == "zero1":
        return PARAM_BF16 + GRAD_BF16 + STATE_F32 / workers
    if method in ("acco", "dpu", "wp"):
        return PARAM_BF16 + GRAD_BF16 + COMM_BF16 + STATE_F32 / workers
    raise ValueError(method)


# algorithmic HBM bytes per element of each entry point (what the operation must move)
BYTES_PER_ELEM = {
    "accumulate": ACCUM_F32 * 2 + GRAD_BF16,            # acc read+write, grad read
    "accumulate_init": ACCUM_F32 + GRAD_BF16,
    "cast": 4 + 2,
    "estimate": 4 * 4 + 2,                              # theta, m, v, gsum read; bf16 out
    "commit": 4 * 4 + 3 * 4,                            # + theta, m, v written
    "commit_bf16": 4 * 4 + 3 * 4 + 2,                   # + fused bf16 parameter output
}


def reduce_bytes_per_elem(workers: int, bf16: bool, accumulate: bool) -> int:
    return workers * (2 if bf16 else 4) + (8 if accumulate else 4)
