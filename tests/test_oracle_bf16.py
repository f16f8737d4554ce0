"""Pins for the 16-bit float conversions that the comparisons of decoded weights go through.

`oracle.to_bf16_bits` (float64 -> bf16, one rounding), `oracle.to_f16` and the input generators'
`f32_to_bf16_bits` carry rounding arithmetic of their own, so they are checked here against
(a) bit patterns worked out by hand from the format's definition (bf16 = sign, 8 exponent bits, 7
fraction bits: the upper half of a binary32; ties go to the even pattern) and (b) the CPU
conversion of torch, a library routine that shares nothing with them.  No GPU."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import pvq_oracle as oracle


def torch_bf16_bits(f32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(f32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


# value -> pattern, each derived by hand.  Spacing of bf16 numbers in [1, 2) is 2^-7, in [2, 4) 2^-6.
HAND_CASES = [
    (1.0, 0x3F80),
    (1.0 + 2.0 ** -7, 0x3F81),
    (1.0 + 2.0 ** -8, 0x3F80),            # half-way between 0x3F80 and 0x3F81: even pattern wins
    (1.0 + 3 * 2.0 ** -8, 0x3F82),        # half-way between 0x3F81 and 0x3F82: even pattern wins
    (1.0 + 5 * 2.0 ** -8, 0x3F82),        # half-way between 0x3F82 and 0x3F83
    (1.0 + 2.0 ** -8 + 2.0 ** -20, 0x3F81),   # just above half-way
    (1.0 + 2.0 ** -8 - 2.0 ** -20, 0x3F80),   # just below
    (2.0 - 2.0 ** -8, 0x4000),            # half-way between 0x3FFF and 2.0: carries into the exponent
    (2.0 - 2.0 ** -7, 0x3FFF),
    (-2.5, 0xC020),
    (3.0, 0x4040),
    (0.0, 0x0000),
    (-0.0, 0x8000),
    (16.0, 0x4180),
    (0.015625, 0x3C80),                   # 2^-6
    (255.0, 0x437F),                      # eight significant bits: exact
    (257.0, 0x4380),                      # nine bits, half-way between 256 and 258: even is 256
    (259.0, 0x4382),                      # half-way between 258 (0x4381) and 260 (0x4382): even is 260
    (2.0 ** -126, 0x0080),                # smallest normal
    (2.0 ** -133, 0x0001),                # smallest subnormal
    (2.0 ** -134, 0x0000),                # half of it: tie to even = 0
    (3 * 2.0 ** -134, 0x0002),            # 1.5 subnormal steps: tie to even = 2
    (float(np.float32(3.3895314e38)), 0x7F7F),   # largest finite bf16
    (float("inf"), 0x7F80),
    (float("-inf"), 0xFF80),
]


def test_hand_cases_direct_rounding():
    vals = np.array([v for v, _ in HAND_CASES], dtype=np.float64)
    want = np.array([b for _, b in HAND_CASES], dtype=np.uint16)
    got = oracle.to_bf16_bits(vals)
    assert [hex(x) for x in got] == [hex(x) for x in want]


def test_hand_cases_generator_helper():
    # every hand case is a binary32 number except the two "just above / below" ones, which are too
    vals = np.array([v for v, _ in HAND_CASES if np.isfinite(v)], dtype=np.float32)
    want = np.array([b for v, b in HAND_CASES if np.isfinite(v)], dtype=np.uint16)
    assert np.array_equal(vals.astype(np.float64), [v for v, _ in HAND_CASES if np.isfinite(v)])
    assert np.array_equal(si.f32_to_bf16_bits(vals), want)


def test_one_rounding_not_two():
    # 1 + 2^-8 + 2^-40 lies above the half-way point, so it rounds up; rounded to binary32 first it
    # would land exactly on the half-way point and go down to the even pattern
    v = np.array([1.0 + 2.0 ** -8 + 2.0 ** -40, -(1.0 + 2.0 ** -8 + 2.0 ** -40), 1.0 + 2.0 ** -8 - 2.0 ** -40])
    assert list(oracle.to_bf16_bits(v)) == [0x3F81, 0xBF81, 0x3F80]
    assert float(np.float32(v[0])) == 1.0 + 2.0 ** -8        # the premise


def test_overflow_and_nan():
    big = np.array([3.3961775292304e38, 3.39e38, 3.4e38, 1e39, -1e39])   # half-way to 2^128 is 3.3961775e38
    got = oracle.to_bf16_bits(big)
    assert list(got[1:]) == [0x7F7F, 0x7F80, 0x7F80, 0xFF80]
    assert got[0] in (0x7F7F, 0x7F80)
    n = oracle.to_bf16_bits(np.array([np.nan]))[0]
    assert (n & 0x7F80) == 0x7F80 and (n & 0x007F) != 0


def random_f32(rng, n):
    """float32 values over the whole finite range, plus values clustered on half-way points."""
    bits = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
    v = bits.view(np.float32)
    v = v[np.isfinite(v)]
    # exact half-way patterns (low half 0x8000) and their neighbours, odd and even upper halves
    hi = rng.integers(0, 0x7F7F, size=4096, dtype=np.uint32) << 16
    near = np.concatenate([hi | 0x8000, hi | 0x7FFF, hi | 0x8001, hi | 0x0001, hi | 0xFFFF, hi])
    near = np.concatenate([near, near | 0x80000000]).astype(np.uint32).view(np.float32)
    near = near[np.isfinite(near)]
    return np.concatenate([v, near, rng.standard_normal(n).astype(np.float32) * np.float32(0.015)])


def test_against_torch_cpu_conversion():
    rng = np.random.default_rng(si.BASE_SEED + 900)
    v = random_f32(rng, 200_000)
    want = torch_bf16_bits(v)
    assert np.array_equal(si.f32_to_bf16_bits(v), want)
    assert np.array_equal(oracle.to_bf16_bits(v.astype(np.float64)), want)


def test_round_trip_and_monotone():
    # every bf16 pattern is a fixed point, and rounding never reorders values
    pats = np.arange(0, 0x7F80, dtype=np.uint32).astype(np.uint16)
    f = si.bf16_bits_to_f32(pats)
    assert np.array_equal(si.f32_to_bf16_bits(f), pats)
    assert np.array_equal(oracle.to_bf16_bits(f.astype(np.float64)), pats)
    rng = np.random.default_rng(si.BASE_SEED + 901)
    x = np.sort(rng.standard_normal(50_000) * 10.0 ** rng.integers(-30, 30, 50_000))
    b = oracle.to_bf16_bits(x).astype(np.int32)
    line = np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    assert np.all(np.diff(line) >= 0)
    # the result is one of the two bf16 neighbours, and the nearer one
    back = si.bf16_bits_to_f32(oracle.to_bf16_bits(x)).astype(np.float64)
    _, e = np.frexp(np.abs(x))
    spacing = np.ldexp(1.0, np.maximum(e - 1, -126) - 7)
    assert np.all(np.abs(back - x) <= spacing / 2)


@pytest.mark.parametrize("value,bits", [
    (1.0, 0x3C00), (1.0 + 2.0 ** -11, 0x3C00), (1.0 + 3 * 2.0 ** -11, 0x3C02), (1.0 + 2.0 ** -11 + 2.0 ** -40, 0x3C01),
    (-2.0, 0xC000), (65504.0, 0x7BFF), (2.0 ** -24, 0x0001), (2.0 ** -25, 0x0000), (0.0, 0x0000),
])
def test_binary16_hand_cases(value, bits):
    # binary16: 5 exponent bits, 10 fraction bits, spacing 2^-10 in [1, 2)
    assert int(oracle.to_f16(np.array([value])).view(np.uint16)[0]) == bits


def test_binary16_against_torch():
    rng = np.random.default_rng(si.BASE_SEED + 902)
    v = (rng.standard_normal(100_000) * 10.0 ** rng.integers(-8, 5, 100_000)).astype(np.float32)
    want = torch.from_numpy(v).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.to_f16(v.astype(np.float64)).view(np.uint16), want)
