"""Host side of the synthetic input generator: distributions, slicing, workload tables."""
import numpy as np

import oracle
import synth


def _f(bits):
    return oracle.bf16_to_f32(bits).astype(np.float64)


def test_slices_are_slices_of_the_full_stream():
    w = synth.WORKLOADS["1b"]
    sp = w.grad_spec(3, 2, 5, 1)
    full = synth.host_grad_bf16(sp, 1000, 5000)
    assert np.array_equal(synth.host_grad_bf16(sp, 3000, 1234), full[2000:3234])
    th = w.host_theta(10, 4000)
    assert np.array_equal(w.host_theta(2010, 100), th[2000:2100])
    # far offsets (beyond 2^31) work
    big = synth.WORKLOADS["7b_hetero"]
    tail = big.host_theta(big.n - 37, 37)
    assert tail.shape == (37,) and np.all(np.isfinite(tail))


def test_streams_differ_by_round_stage_worker_and_microbatch():
    w = synth.WORKLOADS["tiny"]
    base = synth.host_grad_bf16(w.grad_spec(0, 1, 0, 0), 0, 4096)
    for args in ((1, 1, 0, 0), (0, 2, 0, 0), (0, 1, 1, 0), (0, 1, 0, 1)):
        other = synth.host_grad_bf16(w.grad_spec(*args), 0, 4096)
        assert np.mean(other == base) < 0.05
    w2 = synth.Workload(name="x", n=w.n, workers=2, rounds=1, seed=1, grad_std=w.grad_std)
    assert np.mean(synth.host_grad_bf16(w2.grad_spec(0, 1, 0, 0), 0, 4096) == base) < 0.05


def test_value_distributions_match_the_recipes():
    n = 1 << 21
    tiny = synth.WORKLOADS["tiny"]
    th = tiny.host_theta(0, n).astype(np.float64)
    assert abs(th).max() < 0.05 and abs(th.mean()) < 1e-4
    assert abs(th.std() - 0.05 / np.sqrt(3)) < 1e-4
    g = _f(synth.host_grad_bf16(tiny.grad_spec(0, 1, 0, 0), 0, n))
    assert abs(g.std() - 1e-3) < 1e-5 and abs(g.mean()) < 5e-6

    gpt = synth.WORKLOADS["gpt2s"]
    n = 768 * 2730
    a = synth.host_grad_bf16(gpt.grad_spec(2, 1, 0, 0), 0, n)
    b = synth.host_grad_bf16(gpt.grad_spec(2, 2, 3, 5), 0, n)
    za, zb = a == 0, b == 0
    assert 0.03 < za.mean() < 0.07
    # the zero runs are a function of the element index only within a round ...
    runs = za.reshape(-1, 768)
    assert np.all(runs.all(axis=1) | (runs.mean(axis=1) < 0.01))
    assert np.array_equal(za.reshape(-1, 768).all(axis=1), zb.reshape(-1, 768).all(axis=1))
    # ... and change from round to round
    c = synth.host_grad_bf16(gpt.grad_spec(3, 1, 0, 0), 0, n)
    assert not np.array_equal(za, c == 0)

    one = synth.WORKLOADS["1b"]
    n = 1 << 21
    g = _f(synth.host_grad_bf16(one.grad_spec(0, 1, 0, 0), 0, n))
    frac = np.mean(np.abs(g) > 4e-4)       # beyond the Irwin-Hall support of the bulk
    assert 0.5e-3 < frac < 1.2e-3
    assert abs(np.std(g[np.abs(g) <= 4e-4]) - 1e-4) < 2e-6
    th = one.host_theta(0, n).astype(np.float64)
    assert abs(th.std() - 0.02) < 1e-4


def test_workload_tables():
    w = synth.WORKLOADS
    assert w["tiny"].n == 1 << 20 and w["tiny"].workers == 2 and w["tiny"].rounds == 3
    assert w["gpt2s"].n * 4 == 124_439_808 and w["gpt2s"].k_fixed == 8
    assert w["1b"].n == 125_000_000 and w["1b"].warm_steps == 100
    assert w["7b"].n == 875_000_000 and w["7b"].workers == 8 and w["7b"].k_fixed == 4
    assert w["7b_hetero"].n == 875_000_037 and w["7b_hetero"].n % 8 == 5
    for r in range(5):
        ks = [w["7b_hetero"].microbatches(r, k) for k in range(8)]
        assert all(2 <= k <= 8 for k in ks) and len(set(ks)) > 1
        assert [w["7b_hetero"].split(r, k) for k in range(8)] == [(k // 2, k - k // 2) for k in ks]
    sl = w["7b_hetero"].sample_slices()
    assert sl[0][0] == 0 and sl[-1][1] == w["7b_hetero"].n
    assert all(a < b for a, b in sl) and all(sl[i][1] <= sl[i + 1][0] for i in range(len(sl) - 1))
    assert sum(b - a for a, b in sl) < 1 << 20


def test_sampled_ranges_cover_every_phase_of_the_layouts():
    """Full-size runs are checked on sampled index ranges; the interior samples must not sit at
    one fixed phase of the state blocks, tiles or vectors."""
    for name in ("gpt2s", "1b", "7b", "7b_hetero"):
        w = synth.WORKLOADS[name]
        sl = w.sample_slices()
        assert sl[0][0] == 0 and sl[-1][1] == w.n                     # head and (ragged) tail
        assert all(a < b for a, b in sl)
        assert all(sl[k][1] <= sl[k + 1][0] for k in range(len(sl) - 1))   # ascending, disjoint
        inner = sl[1:-1]
        assert len(inner) >= 8
        hit = np.zeros(8192, bool)
        for a, b in inner:
            hit[np.arange(a, b) % 8192] = True
        assert hit.all()                                              # every in-block offset
        starts = {a % 256 for a, _ in inner}
        assert len(starts) == len(inner) if len(inner) <= 256 else len(starts) == 256
        straddle = sum((a // 8192) != ((b - 1) // 8192) for a, b in inner)
        assert straddle >= len(inner) // 3                            # state-block boundaries
        assert any(a % 4 for a, _ in inner) and any(a % 8 == 0 for a, _ in inner)
        assert sum(b - a for a, b in sl) < 400_000                    # the oracle's share stays small
    # the interleaved state buffer (16 bytes per element index) passes 2^32 bytes at element
    # 2^28: samples on both sides of it in the two largest workloads
    for name in ("7b", "7b_hetero"):
        inner = synth.WORKLOADS[name].sample_slices()[1:-1]
        assert any(b < (1 << 28) for _, b in inner) and sum(a > (1 << 28) for a, _ in inner) > 20
    # small shards are checked whole
    assert synth.WORKLOADS["tiny"].sample_slices() == [(0, 1 << 20)]
