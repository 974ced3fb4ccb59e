"""Pins for the oracle's accumulate and reduce (exact sums, numpy fp32 adds, error bounds)."""
import numpy as np
import pytest

import oracle


def _bf16_of_small_ints(rng, n, lo=-64, hi=64):
    """bf16 bit patterns of small integers: exactly representable, sums exact in fp32."""
    ints = rng.integers(lo, hi, size=n)
    bits = (ints.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(oracle.bf16_to_f32(bits), ints.astype(np.float32))
    return ints, bits


@pytest.mark.parametrize("n", [0, 1, 7, 1000, 65537])
def test_accumulate_integer_gradients_sum_exactly(n):
    rng = np.random.default_rng(n)
    acc = np.full(n, 123.0, np.float32)  # garbage that init must overwrite
    total = np.zeros(n, np.int64)
    for k in range(6):
        ints, bits = _bf16_of_small_ints(rng, n)
        oracle.accumulate(acc, bits, init=(k == 0))
        total += ints
    assert np.array_equal(acc, total.astype(np.float32))


def test_accumulate_matches_numpy_fp32_adds_and_fp64_bound():
    rng = np.random.default_rng(3)
    n = 200_003
    acc = np.zeros(n, np.float32)
    ref32 = np.zeros(n, np.float32)
    ref64 = np.zeros(n, np.float64)
    mag = np.zeros(n, np.float64)
    for k in range(8):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        bits = (g.view(np.uint32) >> 16).astype(np.uint16)   # truncation: any bf16 value will do
        gf = oracle.bf16_to_f32(bits)
        oracle.accumulate(acc, bits, init=(k == 0))
        ref32 = gf.copy() if k == 0 else (ref32 + gf).astype(np.float32)
        ref64 += gf.astype(np.float64)
        mag += np.abs(gf.astype(np.float64))
    assert np.array_equal(acc.view(np.uint32), ref32.view(np.uint32))
    # standard recursive-summation bound: |err| <= (k-1) u sum|x|
    assert np.all(np.abs(acc - ref64) <= 7 * 2.0 ** -24 * mag * 1.01 + 1e-45)


def test_accumulate_init_keeps_negative_zero():
    bits = np.array([0x8000, 0x0000], np.uint16)
    acc = np.ones(2, np.float32)
    oracle.accumulate(acc, bits, init=True)
    assert acc.view(np.uint32).tolist() == [0x80000000, 0x00000000]


@pytest.mark.parametrize("W", [1, 2, 3, 8])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_reduce_integer_shards_sum_exactly_and_order_free(W, dtype):
    rng = np.random.default_rng(10 * W)
    n = 4099
    ints, shards = [], []
    for _ in range(W):
        i, b = _bf16_of_small_ints(rng, n)
        ints.append(i)
        shards.append(b if dtype == "bf16" else i.astype(np.float32))
    gsum = np.full(n, -5.0, np.float32)
    oracle.reduce(gsum, shards, accumulate_=False)
    want = np.sum(ints, axis=0)
    assert np.array_equal(gsum, want.astype(np.float32))
    # any worker order gives the same bits when every partial sum is exact
    g2 = np.empty(n, np.float32)
    oracle.reduce(g2, shards[::-1], accumulate_=False)
    assert np.array_equal(g2.view(np.uint32), gsum.view(np.uint32))
    # stage 2: add a second set onto the retained sum
    oracle.reduce(gsum, shards, accumulate_=True)
    assert np.array_equal(gsum, (2 * want).astype(np.float32))


def test_reduce_is_left_to_right_in_worker_order():
    # 2^24 + 1 + 1: left-to-right loses both ones, any other order keeps them
    a = np.array([2.0 ** 24], np.float32)
    one = np.array([1.0], np.float32)
    g = np.empty(1, np.float32)
    oracle.reduce(g, [a, one, one], accumulate_=False)
    assert g[0] == np.float32(2.0 ** 24)
    oracle.reduce(g, [one, one, a], accumulate_=False)
    assert g[0] == np.float32(2.0 ** 24 + 2)
    # accumulate: (((gsum + x0) + x1) ...
    g[0] = 2.0 ** 24
    oracle.reduce(g, [one, one], accumulate_=True)
    assert g[0] == np.float32(2.0 ** 24)


def test_reduce_matches_numpy_fp32_chain_on_random_bf16():
    rng = np.random.default_rng(5)
    n, W = 100_001, 8
    shards = [(rng.standard_normal(n).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
              for _ in range(W)]
    gsum = np.empty(n, np.float32)
    oracle.reduce(gsum, shards, accumulate_=False)
    ref = oracle.bf16_to_f32(shards[0]).copy()
    for w in range(1, W):
        ref = (ref + oracle.bf16_to_f32(shards[w])).astype(np.float32)
    assert np.array_equal(gsum.view(np.uint32), ref.view(np.uint32))
    oracle.reduce(gsum, shards, accumulate_=True)
    for w in range(W):
        ref = (ref + oracle.bf16_to_f32(shards[w])).astype(np.float32)
    assert np.array_equal(gsum.view(np.uint32), ref.view(np.uint32))


def test_reduce_first_term_keeps_negative_zero():
    s = [np.array([0x8000], np.uint16), np.array([0x8000], np.uint16)]
    g = np.ones(1, np.float32)
    oracle.reduce(g, s, accumulate_=False)
    assert g.view(np.uint32)[0] == 0x80000000
