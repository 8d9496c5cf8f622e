"""Pins of the bf16 widening that every bf16 parity claim rests on.

The expected values are hand-written from the format itself (1 sign, 8 exponent, 7 fraction bits;
value = (-1)^s 2^(e-127) (1 + f/128), subnormal 2^-126 f/128) and from Python's own float32 packing
(struct), not from the functions under test.  The seeded generator's rounding to bf16 (round to
nearest, ties to even) is pinned the same way, including tie cases in both directions.
"""
import math
import struct

import numpy as np

from oracle import vmonarch_oracle as O
from paper_2601_22275_amd import synth

# (bit pattern, exact value)
HAND = [
    (0x3F80, 1.0),
    (0xBF80, -1.0),
    (0xC000, -2.0),
    (0x4000, 2.0),
    (0x3EAB, 0.333984375),            # 2^-2 * (1 + 43/128)
    (0x3F00, 0.5),
    (0x4049, 3.140625),               # 2^1 * (1 + 73/128)
    (0x42F7, 123.5),                  # 2^6 * (1 + 119/128)
    (0x7F7F, (2.0 - 2.0 ** -7) * 2.0 ** 127),   # largest finite
    (0x0080, 2.0 ** -126),            # smallest normal
    (0x0001, 2.0 ** -133),            # smallest subnormal: 2^-126 / 128
    (0x0040, 2.0 ** -127),            # subnormal with the top fraction bit
    (0x8001, -(2.0 ** -133)),
    (0x0000, 0.0),
    (0x8000, -0.0),
]


def test_widen_bf16_hand_written_patterns():
    bits = np.array([b for b, _ in HAND], dtype=np.uint16)
    got = O.widen_bf16(bits)
    assert got.dtype == np.float64
    for (pattern, want), g in zip(HAND, got):
        assert g == want, (hex(pattern), g, want)
        assert math.copysign(1.0, g) == math.copysign(1.0, want), hex(pattern)   # the sign of zero too


def test_widen_bf16_special_values():
    got = O.widen_bf16(np.array([0x7F80, 0xFF80, 0x7FC0], dtype=np.uint16))
    assert got[0] == math.inf and got[1] == -math.inf and math.isnan(got[2])


def test_widen_bf16_is_the_upper_half_of_a_float32_for_every_pattern():
    """All 65,536 patterns against struct's float32 decoding of (pattern << 16)."""
    bits = np.arange(1 << 16, dtype=np.uint32)
    with np.errstate(invalid="ignore"):             # the table holds signalling-NaN patterns
        got = O.widen_bf16(bits.astype(np.uint16))
    for p in range(0, 1 << 16, 97):                 # struct, one by one, on a stride that hits every exponent
        want = struct.unpack("<f", struct.pack("<I", p << 16))[0]
        g = float(got[p])
        assert (math.isnan(want) and math.isnan(g)) or g == want, hex(p)
    # and the whole table against the format's definition, for the finite normal patterns
    s = (bits >> 15) & 1
    e = ((bits >> 7) & 0xFF).astype(np.int64)
    f = (bits & 0x7F).astype(np.float64)
    normal = (e > 0) & (e < 255)
    want = np.where(s == 1, -1.0, 1.0) * np.ldexp(1.0 + f / 128.0, (e - 127).astype(np.int32))
    assert np.array_equal(got[normal], want[normal])
    sub = e == 0
    want_sub = np.where(s == 1, -1.0, 1.0) * f / 128.0 * 2.0 ** -126
    assert np.array_equal(got[sub], want_sub[sub])


def test_widen_bf16_keeps_shape_and_accepts_any_uint16_layout():
    x = np.array([[0x3F80, 0xC000], [0x3EAB, 0x0000]], dtype=np.uint16)
    got = O.widen_bf16(x)
    assert got.shape == (2, 2)
    assert np.array_equal(got, np.array([[1.0, -2.0], [0.333984375, 0.0]]))
    assert np.array_equal(O.widen_bf16(x.T.copy()), got.T)
    assert np.array_equal(O.widen_bf16(x[:, ::-1]), got[:, ::-1])      # a strided view


# ---------------------------------------------------------------- the generator's rounding to bf16
def test_generator_rounding_ties_to_even_and_round_trip():
    # 1 + 2^-8 lies exactly between 0x3F80 (even) and 0x3F81: goes down to even;
    # 1 + 3 * 2^-8 lies exactly between 0x3F81 and 0x3F82 (even): goes up to even.
    cases = [
        (1.0, 0x3F80),
        (1.0 + 2.0 ** -8, 0x3F80),
        (1.0 + 3.0 * 2.0 ** -8, 0x3F82),
        (1.0 + 2.0 ** -8 + 2.0 ** -20, 0x3F81),      # just above the tie: up
        (1.0 + 2.0 ** -8 - 2.0 ** -20, 0x3F80),      # just below: down
        (-(1.0 + 3.0 * 2.0 ** -8), 0xBF82),
        (0.333984375, 0x3EAB),                       # already representable
        (1.0 / 3.0, 0x3EAB),                         # 0.33333 -> 0x3EAB (0.33398), nearer than 0x3EAA (0.33203)
        (0.0, 0x0000),
        (-0.0, 0x8000),
        (float(np.float32(3.3895314e38)), 0x7F7F),   # top finite bf16 + less than half an ulp stays finite
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    got = synth.f32_to_bf16_bits(x)
    assert got.dtype == np.uint16
    for (val, want), g in zip(cases, got):
        assert int(g) == want, (val, hex(int(g)), hex(want))
    # every bf16 value survives widen -> float32 -> round
    allbits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    e = (allbits >> 7) & 0xFF
    finite = allbits[e != 0xFF]
    assert np.array_equal(synth.f32_to_bf16_bits(O.widen_bf16(finite).astype(np.float32)), finite)
    # and the generator's own narrowing inverse agrees with the oracle's widening
    assert np.array_equal(synth.bf16_bits_to_f32(finite).astype(np.float64), O.widen_bf16(finite))


def test_generator_rounding_is_nearest_on_random_values():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    w = O.widen_bf16(bits)
    up = O.widen_bf16((bits + 1).astype(np.uint16))
    dn = O.widen_bf16((bits - 1).astype(np.uint16))
    x64 = x.astype(np.float64)
    err = np.abs(w - x64)
    ok = np.isfinite(up) & np.isfinite(dn)
    assert (err[ok] <= np.abs(up[ok] - x64[ok])).all() and (err[ok] <= np.abs(dn[ok] - x64[ok])).all()
