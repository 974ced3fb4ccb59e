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


# ---------------------------------------------------------------- bf16 running sum (paper Sec. 4)

def _bf16_value(bits: int):
    """Exact rational value of a finite bf16 bit pattern."""
    from fractions import Fraction
    sign = -1 if bits & 0x8000 else 1
    e, f = (bits >> 7) & 0xFF, bits & 0x7F
    if e == 0:
        return sign * Fraction(f, 1 << 7) * Fraction(2) ** -126
    return sign * (1 + Fraction(f, 1 << 7)) * Fraction(2) ** (e - 127)


def _nearest_even_bf16(x):
    """Round an exact rational to bf16, ties to even, by searching the neighbours."""
    from fractions import Fraction
    if x == 0:
        return None                         # sign of zero decided by IEEE rules, checked apart
    sign, a = (0x8000 if x < 0 else 0), abs(x)
    lo, hi = 0, 0x7F7F                      # magnitudes of finite bf16 patterns are monotone
    while lo < hi:                          # largest pattern with value <= a
        mid = (lo + hi + 1) // 2
        if _bf16_value(mid) <= a:
            lo = mid
        else:
            hi = mid - 1
    below = _bf16_value(lo)
    if below == a or lo == 0x7F7F:
        return sign | lo
    above = _bf16_value(lo + 1)
    if a - below < above - a or (a - below == above - a and lo % 2 == 0):
        return sign | lo
    return sign | (lo + 1)


def test_accumulate_bf16_is_the_correctly_rounded_bf16_sum():
    rng = np.random.default_rng(11)
    n = 4000
    # exponents close together so that the sum needs rounding, plus cancellation and subnormals
    e = rng.integers(100, 140, size=n)
    a = ((rng.integers(0, 2, n) << 15) | (e << 7) | rng.integers(0, 128, n)).astype(np.uint16)
    b = ((rng.integers(0, 2, n) << 15) | ((e + rng.integers(-9, 10, n)) << 7)
         | rng.integers(0, 128, n)).astype(np.uint16)
    a[:50] = rng.integers(0, 0x0100, 50)                 # subnormal and tiny values
    b[:50] = rng.integers(0, 0x0100, 50) | 0x8000
    acc = a.copy()
    oracle.accumulate_bf16(acc, b, init=False)
    checked = 0
    for j in range(n):
        want = _nearest_even_bf16(_bf16_value(int(a[j])) + _bf16_value(int(b[j])))
        if want is None:
            assert acc[j] & 0x7FFF == 0
            continue
        assert int(acc[j]) == want, (hex(a[j]), hex(b[j]), hex(acc[j]), hex(want))
        checked += 1
    assert checked > 3900


def test_accumulate_bf16_matches_torch_bf16_add_and_init_copies():
    import torch
    rng = np.random.default_rng(12)
    n = 100_003
    g = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(5)]
    bits = [(x.view(np.uint32) >> 16).astype(np.uint16) for x in g]
    acc = np.full(n, 0x4123, np.uint16)
    ref = None
    for k, b in enumerate(bits):
        oracle.accumulate_bf16(acc, b, init=(k == 0))
        t = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16)
        ref = t.clone() if k == 0 else ref + t           # library bf16 add
        if k == 0:
            assert np.array_equal(acc, b)
    assert np.array_equal(acc.view(np.int16), ref.view(torch.int16).numpy())


def test_accumulate_bf16_stagnates_at_256_where_fp32_does_not():
    """8 significand bits: 256 + 1 is a tie that rounds to even (256), so a bf16 running sum of
    ones stops growing at 256; the fp32 accumulator reaches the exact count."""
    one = np.full(3, 0x3F80, np.uint16)
    acc16 = np.zeros(3, np.uint16)
    acc32 = np.zeros(3, np.float32)
    for k in range(300):
        oracle.accumulate_bf16(acc16, one, init=(k == 0))
        oracle.accumulate(acc32, one, init=(k == 0))
    assert np.all(oracle.bf16_to_f32(acc16) == 256.0)
    assert np.all(acc32 == 300.0)
