"""Buffers placed by memory class: the classification call, the arena that hands out tensors by
class, and whole rounds on arena-placed buffers (placement changes no bit)."""
import pytest

import synth
from test_gpu_rounds import run_workload

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

GiB = 1 << 30


def log(*a):
    print(*a, flush=True)


def test_classification_labels_every_position_and_repeats():
    import paper_2406_02613_amd as A
    B = A.binding
    free = torch.cuda.mem_get_info()[0]
    size = min(200 * GiB, int(0.7 * free)) // GiB * GiB
    region = torch.empty(size, dtype=torch.uint8, device="cuda")
    scratch = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    def one_pass(rep):
        classes, ncls = B.acco_hbm_classify(region, 2 * GiB, 512 << 20, scratch)
        log(f"classification {rep}: {size // GiB} GiB, {ncls} classes:",
            "".join(str(c) if c < 10 else "+" for c in classes))
        assert len(classes) == (size - (512 << 20)) // (2 * GiB) + 1
        assert 1 <= ncls <= 64 and set(classes) == set(range(ncls))
        sizes = [classes.count(c) for c in range(ncls)]
        assert sizes == sorted(sizes, reverse=True)          # numbered by size, largest first
        return classes

    def agreement(a, b):
        # do two passes partition the positions the same way?  (Class numbers may swap where two
        # classes are equally large, so compare which pairs of neighbours share a class.)
        same = [(a0 == a1) == (b0 == b1) for a0, a1, b0, b1 in zip(a, a[1:], b, b[1:])]
        return sum(same) / max(1, len(same))

    # the classification is a timing measurement: other work on the device can disturb one
    # pass, so a third is taken before two passes are said to disagree
    runs = [one_pass(0), one_pass(1)]
    if agreement(runs[0], runs[1]) < 0.9:
        runs.append(one_pass(2))
    best = max(agreement(a, b) for i, a in enumerate(runs) for b in runs[i + 1:])
    assert best >= 0.9, f"no two of {len(runs)} passes agree: {best:.2f}"
    # the region is only read, the scratch written
    with pytest.raises(A.AccoError):
        B.acco_hbm_classify(region, 2 * GiB, 512 << 20, region[:512 << 20])


def test_arena_hands_out_aligned_tensors_of_the_requested_class():
    import paper_2406_02613_amd as A
    arena = A.HbmArena(6 * GiB, step_bytes=GiB, probe_bytes=256 << 20)
    log("arena:", arena.describe())
    assert arena.n_classes >= 1 and sum(arena.free_bytes().values()) > 4 * GiB
    t = arena.alloc(1000, torch.float32, 0, zero=True)
    u = arena.alloc(1 << 20, torch.bfloat16, 0)
    assert t.dtype == torch.float32 and t.numel() == 1000 and not t.any()
    assert t.data_ptr() % (1 << 21) == 0 and u.data_ptr() % (1 << 21) == 0
    assert u.data_ptr() >= t.data_ptr() + (1 << 21)
    assert t.acco_class == 0 and u.acco_class == 0
    with pytest.raises(MemoryError):
        arena.alloc(7 * GiB, torch.uint8, 0)
    t.fill_(3.0)
    u.zero_()
    torch.cuda.synchronize()
    assert float(t.sum()) == 3000.0                        # neighbours do not overlap


def test_rounds_on_arena_placed_buffers_change_no_bits():
    import paper_2406_02613_amd as A
    arena = A.HbmArena(8 * GiB, step_bytes=GiB, probe_bytes=256 << 20)
    w = synth.WORKLOADS["tiny"]
    owner = run_workload(w, fused_publish=True, fused_reduce=True, blocked=True, stash=True,
                         batched=True, arena=arena)
    g = owner.new_gradient_buffer()
    assert g.dtype == torch.bfloat16 and g.numel() == w.n
    run_workload(w, arena=arena, rounds=2)                                    # planar state
    run_workload(w, arena=arena, rounds=2, interleaved=True, stash=True, fused_publish=True,
                 fused_reduce=True, batched=True)
    ragged = synth.Workload(name="ragged_arena", n=300_037, workers=3, rounds=2, grad_std=1e-3,
                            k_range=(2, 6), seed=31)
    run_workload(ragged, arena=arena, fused_publish=True, fused_reduce=True, blocked=True,
                 stash=True, batched=True, dev_scalars=True)
