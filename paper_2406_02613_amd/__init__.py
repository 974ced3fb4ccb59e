"""ACCO per-shard optimizer path for AMD MI355X: HIP kernels behind a C ABI, and a thin binding."""
from .binding import (ACCO_BF16, ACCO_F32, AccoError, AdamW, Counter, acco_accumulate,
                      acco_accumulate_bf16, acco_accumulate_batch,
                      acco_accumulate_first, acco_accumulate_publish, acco_accumulate_second,
                      acco_cast_params, acco_commit_step,
                      acco_estimate_step, acco_lr_cosine, acco_reduce_commit_step, acco_reduce_estimate_step,
                      acco_reduce_shards, acco_sgd_commit_step, acco_sgd_estimate_step, make_sgd,
                      Sgd,
                      make_hyper, set_launch_shape, set_resident_waves, reset_launch_settings,
                      status_string,
                      version)
from .shard import RecordedRound, ShardOwner
from .state import BlockedState, InterleavedShards
from .arena import HbmArena
from .two_stream import TwoStreamOwner
from .schemes import SchemeOwner, SCHEMES
from . import layout

__all__ = ["ACCO_BF16", "ACCO_F32", "AccoError", "AdamW", "Counter", "acco_accumulate",
           "acco_accumulate_bf16", "acco_accumulate_batch",
           "acco_accumulate_first", "acco_accumulate_publish", "acco_accumulate_second",
           "acco_cast_params", "acco_commit_step", "acco_estimate_step",
           "acco_lr_cosine", "acco_reduce_commit_step", "acco_reduce_estimate_step", "acco_reduce_shards",
           "acco_sgd_commit_step", "acco_sgd_estimate_step", "make_sgd", "Sgd", "SchemeOwner", "SCHEMES", "BlockedState", "InterleavedShards", "TwoStreamOwner",
           "make_hyper", "set_launch_shape", "set_resident_waves", "reset_launch_settings", "status_string", "version", "ShardOwner", "RecordedRound", "HbmArena", "layout"]
