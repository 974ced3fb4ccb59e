"""Host-side logic of bench.py that needs no GPU: the refusal of more than one GPU, the table of
algorithmic bytes per element behind every roofline figure, and the mapping from profiler
dispatches to bench labels."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in (r.stdout + r.stderr)
    assert "{" not in r.stdout                      # no result line


# bytes per shard element and launch, counted by hand from what each kernel reads and writes
# (fp32 = 4, bf16 = 2; state = theta, m, v; W bf16 shards for the reductions)
@pytest.mark.parametrize("label,W,want", [
    ("commit", 8, 4 * 4 + 3 * 4),                   # theta, m, v, gsum in; theta, m, v out
    ("commit_bf16", 8, 4 * 4 + 3 * 4 + 2),
    ("estimate", 8, 4 * 4 + 2),
    ("accumulate", 8, 4 + 2 + 4),
    ("accumulate_init", 8, 2 + 4),
    ("cast", 8, 4 + 2),
    ("reduce_init", 8, 8 * 2 + 4),
    ("reduce_accumulate", 8, 8 * 2 + 4 + 4),
    ("reduce_init", 3, 3 * 2 + 4),
    ("reduce_estimate", 8, 3 * 4 + 8 * 2 + 4 + 2),
    ("reduce_commit_bf16", 8, 4 * 4 + 8 * 2 + 3 * 4 + 2),
    ("reduce_commit_bf16@dev", 8, 46),
    ("accumulate_first*8", 8, 8 * 4),
    ("accumulate_second_publish*8", 8, 8 * 6),
    ("accumulate_second*3", 8, 3 * 8),
    ("accumulate_publish*5", 8, 5 * 8),
])
def test_algorithmic_bytes_per_element(label, W, want):
    assert bench.kernel_bytes_per_elem(label, W) == want


def test_default_round_moves_240_bytes_per_element():
    # two micro-batches per worker and stage at W = 8: stash + (second, publish) per stage, then
    # the fused reduce + estimate and reduce + commit
    per_stage = bench.kernel_bytes_per_elem("accumulate_first*8", 8) + \
        bench.kernel_bytes_per_elem("accumulate_second_publish*8", 8)
    total = 2 * per_stage + bench.kernel_bytes_per_elem("reduce_estimate", 8) + \
        bench.kernel_bytes_per_elem("reduce_commit_bf16", 8)
    assert total == 240


def test_dispatch_labels():
    n = 875_000_037
    lanes = -(-(n // 8) // 64) * 64                 # work-items of one worker's row, 8 per lane
    stash = ("void acco::flat_kernel<acco::Batch<acco::StashOp<false, false> > >"
             "(acco::Batch<acco::StashOp<false, false> >, long)")
    assert bench._label_of(stash, 8 * lanes, n) == "accumulate_first*8"
    assert bench._label_of(stash, 3 * lanes, n) == "accumulate_first*3"
    assert bench._label_of("hipMemcpy something else", 64, n) is None
    short = bench._short_kernel(stash)
    assert "StashOp" in short and "(" not in short
