"""Pins for the oracle's bf16 <-> fp32 conversions (none of them calls the oracle's own formula)."""
import os

import numpy as np
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bf16_rne_cases.txt")


def _cast_bits(u32: np.ndarray) -> np.ndarray:
    return oracle.cast(np.ascontiguousarray(u32.astype(np.uint32)).view(np.float32))


def test_hand_worked_rounding_cases():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 20
    src = np.array([int(r[0], 16) for r in rows], dtype=np.uint32)
    want = np.array([int(r[1], 16) for r in rows], dtype=np.uint16)
    got = _cast_bits(src)
    bad = [(rows[i][0], rows[i][1], hex(got[i])) for i in range(len(rows)) if got[i] != want[i]]
    assert not bad, bad
    # the scalar entry point agrees with the array one
    for r in rows:
        f = np.array([int(r[0], 16)], dtype=np.uint32).view(np.float32)[0]
        assert oracle.lib().oracle_f32_to_bf16(float(f)) == int(r[1], 16)


def test_widening_is_the_high_half_for_all_65536_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.lib().oracle_bf16_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def test_round_trip_identity_for_all_bf16_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    f = oracle.bf16_to_f32(bits)
    back = oracle.cast(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], bits[~nan])
    # NaNs stay NaNs with their sign
    assert np.all((back[nan] & 0x7F80) == 0x7F80) and np.all((back[nan] & 0x007F) != 0)
    assert np.array_equal(back[nan] & 0x8000, bits[nan] & 0x8000)


def test_against_torch_cpu_cast_on_random_and_boundary_patterns():
    rng = np.random.default_rng(1234)
    rnd = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    # every bf16 value with every "interesting" low half: below / at / above the tie
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    grid = (hi[:, None] | lows[None, :]).ravel()
    src = np.concatenate([rnd, grid])
    got = _cast_bits(src)
    t = torch.from_numpy(src.view(np.int32)).view(torch.float32).to(torch.bfloat16)
    want = t.view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(src.view(np.float32))
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x007F) != 0)


def test_rounding_error_is_at_most_half_a_bf16_ulp():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(500_000) * np.exp(rng.uniform(-20, 20, 500_000))).astype(np.float32)
    y = oracle.bf16_to_f32(oracle.cast(x)).astype(np.float64)
    # ulp of bf16 at x: 2^(exponent - 7)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(x.astype(np.float64)))) - 7)
    assert np.all(np.abs(y - x) <= 0.5 * ulp * (1 + 1e-12))
