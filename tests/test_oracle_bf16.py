"""Pin for oracle.decode_bf16, through which every bfloat16 input enters the oracle.

bfloat16 is the upper half of an IEEE binary32: 1 sign bit, 8 exponent bits (bias 127), 7 fraction
bits.  The checks below do not call the oracle's own shift: they use the format's definition written
out with integer arithmetic, hand-written bit patterns, and torch's bfloat16 type (a library routine).
"""
import math

import numpy as np
import torch

from oracle import moe_oracle as O


def value_from_fields(bits: int) -> float:
    """sign, exponent and fraction fields -> value, by the format's definition."""
    sign = -1.0 if bits & 0x8000 else 1.0
    exp = (bits >> 7) & 0xFF
    frac = bits & 0x7F
    if exp == 0xFF:
        return sign * math.inf if frac == 0 else math.nan
    if exp == 0:
        return sign * math.ldexp(frac, -126 - 7)           # zero and subnormals
    return sign * math.ldexp(128 + frac, exp - 127 - 7)


def test_hand_written_patterns():
    cases = {
        0x3F80: 1.0,
        0xC020: -2.5,
        0x0000: 0.0,
        0x8000: -0.0,
        0x0001: 2.0 ** -133,          # smallest subnormal
        0x007F: 127 * 2.0 ** -133,    # largest subnormal
        0x0080: 2.0 ** -126,          # smallest normal
        0x7F7F: (2.0 - 2.0 ** -7) * 2.0 ** 127,   # largest finite
        0x3DCD: 0.10009765625,        # 0.1 rounded to nearest even
        0x4049: 3.140625,             # pi rounded
        0xBF00: -0.5,
    }
    bits = np.array(list(cases), dtype=np.uint16)
    got = O.decode_bf16(bits)
    assert got.dtype == np.float64
    for b, g in zip(cases, got):
        assert g == cases[b], (hex(b), g, cases[b])
    assert math.copysign(1.0, got[3]) == -1.0 and math.copysign(1.0, got[2]) == 1.0
    assert O.decode_bf16(np.array([0x7F80, 0xFF80], dtype=np.uint16)).tolist() == [math.inf, -math.inf]
    assert np.all(np.isnan(O.decode_bf16(np.array([0x7F81, 0x7FC0, 0xFFFF], dtype=np.uint16))))


def test_all_patterns_against_the_format_definition_and_torch():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = O.decode_bf16(bits)
    want = np.array([value_from_fields(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # torch's bfloat16 widened by the library
    tv = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    assert np.array_equal(np.isnan(tv), nan)
    assert np.array_equal(got[~nan], tv[~nan])
    # fp32 variant and shape handling
    g32 = O.decode_bf16(bits.reshape(256, 256), dtype=np.float32)
    assert g32.shape == (256, 256) and g32.dtype == np.float32
    assert np.array_equal(g32.reshape(-1)[~nan].astype(np.float64), want[~nan])


def test_rounded_inputs_survive_a_round_trip():
    """Values that are exactly representable (8 significant bits) decode to themselves."""
    rng = np.random.default_rng(0)
    m = rng.integers(128, 256, size=1000)           # 8-bit significands
    e = rng.integers(-30, 30, size=1000)
    s = rng.choice([-1.0, 1.0], size=1000)
    vals = s * np.ldexp(m.astype(np.float64), e - 7)
    bits = (vals.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)   # exact: low 16 bits are zero
    assert np.all((vals.astype(np.float32).view(np.uint32) & 0xFFFF) == 0)
    assert np.array_equal(O.decode_bf16(bits), vals)
