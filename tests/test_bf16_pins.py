"""Pins of the bf16 <-> fp32/fp64 conversions that carry every test input and
every compared output: the oracle's widening and the input generator's
round-to-nearest-even narrowing, each against an independent implementation
(torch's bf16 cast, and the format's definition evaluated with Python
integers/`math.ldexp`).  CPU only."""
import math
import struct

import numpy as np
import torch

from oracle import ref_numpy as rn
from paper_2604_27089_amd import synth

ALL = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)


def decode_bf16(bits: int) -> float:
    """bf16 = 1 sign, 8 exponent (bias 127), 7 fraction bits, from the format's definition."""
    sign = -1.0 if bits >> 15 else 1.0
    e, f = (bits >> 7) & 0xFF, bits & 0x7F
    if e == 0xFF:
        return sign * math.inf if f == 0 else math.nan
    if e == 0:
        return sign * math.ldexp(f, -126 - 7)
    return sign * math.ldexp(128 + f, e - 127 - 7)


def test_widen_all_patterns_against_torch():
    t = torch.from_numpy(ALL.view(np.int16)).view(torch.bfloat16)
    for got in (rn.widen_bf16(ALL), synth.bf16_bits_to_f32(ALL).astype(np.float64)):
        want = t.to(torch.float64).numpy()
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got[~nan], want[~nan])
        assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))  # -0.0 stays -0.0


def test_widen_all_patterns_against_the_format_definition():
    got = rn.widen_bf16(ALL)
    for b in range(0, 1 << 16, 7):  # every 7th pattern plus the special ones below
        w = decode_bf16(b)
        assert (math.isnan(w) and math.isnan(got[b])) or got[b] == w, hex(b)
    for b in (0x0000, 0x8000, 0x0001, 0x007F, 0x0080, 0x3F80, 0xBF80, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80, 0x7FC0):
        w = decode_bf16(b)
        assert (math.isnan(w) and math.isnan(got[b])) or got[b] == w, hex(b)
    assert got[0x3F80] == 1.0 and got[0x4000] == 2.0 and got[0xC040] == -3.0
    assert got[0x7F7F] == (2.0 - 2.0 ** -7) * 2.0 ** 127  # largest finite value


def test_narrow_roundtrip_is_identity_on_every_pattern():
    wide = synth.bf16_bits_to_f32(ALL)
    back = synth.f32_to_bf16_bits(wide)
    nan = np.isnan(wide)
    assert np.array_equal(back[~nan], ALL[~nan])
    assert np.all(np.isnan(synth.bf16_bits_to_f32(back[nan])))


def test_narrow_random_values_against_torch():
    rng = np.random.default_rng(5)
    x = np.concatenate([
        rng.standard_normal(1 << 20, dtype=np.float32),
        (rng.standard_normal(1 << 18, dtype=np.float32) * np.float32(1e-30)),
        (rng.standard_normal(1 << 18, dtype=np.float32) * np.float32(1e30)),
        rng.integers(0, 1 << 32, 1 << 20, dtype=np.uint64).astype(np.uint32).view(np.float32),  # any bit pattern
    ])
    got = synth.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all(np.isnan(synth.bf16_bits_to_f32(got[nan])))


def f32(bits: int) -> np.float32:
    return np.frombuffer(struct.pack("<I", bits), dtype=np.float32)[0]


def test_narrow_ties_and_special_values():
    cases = {
        # exact ties: the discarded half is exactly 0x8000 -> round to the even neighbour
        0x3F808000: 0x3F80,  # 1 + 2^-8  -> 1 (even)
        0x3F818000: 0x3F82,  # 1 + 3*2^-8 -> 1 + 2^-6 (even)
        0xBF808000: 0xBF80,
        0xBF818000: 0xBF82,
        # just below / above a tie
        0x3F807FFF: 0x3F80,
        0x3F808001: 0x3F81,
        # carry into the exponent, and into infinity from the largest finite fp32 values
        0x3FFFFFFF: 0x4000,
        0x7F7FFFFF: 0x7F80,
        0x7F7F7FFF: 0x7F7F,  # stays the largest finite bf16
        0x7F7F8000: 0x7F80,  # tie between largest finite (odd) and infinity -> even = infinity
        # infinities and zeros
        0x7F800000: 0x7F80, 0xFF800000: 0xFF80, 0x00000000: 0x0000, 0x80000000: 0x8000,
        # subnormals: fp32 subnormal below half the smallest bf16 subnormal -> 0; tie -> even (0)
        0x00000001: 0x0000, 0x00008000: 0x0000, 0x00008001: 0x0001, 0x00018000: 0x0002,
        0x007FFFFF: 0x0080,  # largest fp32 subnormal rounds up to the smallest normal
    }
    x = np.array([f32(b) for b in cases], dtype=np.float32)
    got = synth.f32_to_bf16_bits(x)
    assert [int(g) for g in got] == list(cases.values())
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # NaNs (quiet, signalling, negative) stay NaN
    nans = np.array([f32(b) for b in (0x7FC00000, 0x7F800001, 0xFFC00001, 0x7FFFFFFF)], dtype=np.float32)
    assert np.all(np.isnan(rn.widen_bf16(synth.f32_to_bf16_bits(nans))))


def test_narrow_is_nearest_and_monotone():
    rng = np.random.default_rng(6)
    x = np.sort(rng.standard_normal(200000, dtype=np.float32) * np.float32(8))
    b = synth.f32_to_bf16_bits(x)
    y = rn.widen_bf16(b)
    assert np.all(np.diff(y) >= 0)
    # error at most half a bf16 ulp of the result's binade
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(y), 2.0 ** -126))) - 7)
    assert np.all(np.abs(y - x.astype(np.float64)) <= 0.5 * ulp)
