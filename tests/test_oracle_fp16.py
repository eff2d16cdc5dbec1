"""Pins for the oracle's bitwise fp16 converters: independent library casts (torch's and
numpy's) over every fp32 and every fp16 bit pattern, plus hand-derived boundary values."""
import numpy as np
import pytest
import torch

import oracle


def _torch_f16_bits(x32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(x32).to(torch.float16).view(torch.int16).numpy().view(np.uint16)


def _check_chunk(x32, want):
    got = oracle.f32_to_f16_bits(x32)
    nan = np.isnan(x32)
    assert np.array_equal(got[~nan], want[~nan])
    if nan.any():  # NaN stays NaN with the sign kept; payload is free
        assert np.all((got[nan] & 0x7C00) == 0x7C00) and np.all((got[nan] & 0x03FF) != 0)
        assert np.array_equal(got[nan] & 0x8000, (x32[nan].view(np.uint32) >> 16).astype(np.uint16) & 0x8000)


def test_f32_to_f16_every_bit_pattern_vs_torch():
    low = np.arange(1 << 24, dtype=np.uint32)
    for hi in range(256):
        x = (low | np.uint32(hi << 24)).view(np.float32)
        _check_chunk(x, _torch_f16_bits(x))


@pytest.mark.parametrize("hi", [0x00, 0x33, 0x38, 0x39, 0x47, 0x7F, 0xB8, 0xFF])
def test_f32_to_f16_vs_numpy_cast(hi):
    # numpy's software cast is slow; cover the zero/subnormal, normal, overflow and NaN blocks
    low = np.arange(0, 1 << 24, 5, dtype=np.uint32)
    x = (low | np.uint32(hi << 24)).view(np.float32)
    with np.errstate(all="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    _check_chunk(x, want)


def test_f16_to_f32_every_bit_pattern_vs_numpy():
    h = np.arange(1 << 16, dtype=np.uint16)
    got = oracle.f16_bits_to_f32(h)
    want = h.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    assert np.all(np.isnan(got[nan]))


def test_roundtrip_f16_f32_f16_is_identity():
    h = np.arange(1 << 16, dtype=np.uint16)
    back = oracle.f32_to_f16_bits(oracle.f16_bits_to_f32(h))
    nan = (h & 0x7C00 == 0x7C00) & (h & 0x3FF != 0)
    assert np.array_equal(back[~nan], h[~nan])


@pytest.mark.parametrize("value,bits", [
    (0.0, 0x0000), (-0.0, 0x8000), (1.0, 0x3C00), (-2.0, 0xC000),
    (65504.0, 0x7BFF),            # largest finite half
    (65519.996, 0x7BFF),          # just below the rounding boundary to infinity
    (65520.0, 0x7C00),            # halfway between 65504 and 2^16: ties-to-even goes up to inf
    (1e9, 0x7C00), (-1e9, 0xFC00),
    (2.0 ** -14, 0x0400),         # smallest normal
    (2.0 ** -24, 0x0001),         # smallest subnormal
    (2.0 ** -25, 0x0000),         # exact tie between 0 and 2^-24 -> even (0)
    (2.0 ** -25 * 1.0000001, 0x0001),
    (3 * 2.0 ** -25, 0x0002),     # tie between 1 and 2 units -> even (2)
    (-(2.0 ** -26), 0x8000),      # underflows to -0, sign kept
    (1.0 + 2.0 ** -11, 0x3C00),   # tie, even mantissa stays
    (1.0 + 3 * 2.0 ** -11, 0x3C02),  # tie, odd mantissa rounds up
    (1.0 + 2.0 ** -11 + 2.0 ** -23, 0x3C01),
    (2.0 ** -14 - 2.0 ** -25, 0x0400),  # largest subnormal + half unit -> tie to even = min normal
])
def test_f32_to_f16_hand_derived(value, bits):
    got = oracle.f32_to_f16_bits(np.array([value], np.float32))[0]
    assert got == bits, hex(got)
