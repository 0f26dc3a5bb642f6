"""Pins for the oracle's storage-format rounding (bf16 and f32), independent of the oracle:
exhaustive round trips, hand-built midpoints, and an exact-rational rounding routine."""
import math
import struct

import numpy as np
import pytest

import oracle
from bruteforce import bf16_bits_to_float, round_to_bf16_bits


def f32_of_bits(u):
    return struct.unpack("<f", struct.pack("<I", u))[0]


def test_all_bf16_patterns_round_trip():
    for b in range(0x10000):
        v = oracle.bf16_to_f64(b)
        if v != v:
            assert oracle.bf16_from_f64(v) & 0x7F80 == 0x7F80
            continue
        assert v == bf16_bits_to_float(b)
        assert oracle.bf16_from_f64(v) == b, hex(b)


def test_bf16_midpoints_go_to_even_and_neighbours_split():
    # every pair of adjacent positive finite bf16 values: the midpoint goes to the even one, and
    # one fp64 ulp either side of the midpoint goes to the nearer one.
    for b in range(0x0000, 0x7F7F):
        lo, hi = oracle.bf16_to_f64(b), oracle.bf16_to_f64(b + 1)
        mid = (lo + hi) / 2            # exact in fp64
        even = b if (b & 1) == 0 else b + 1
        assert oracle.bf16_from_f64(mid) == even, hex(b)
        assert oracle.bf16_from_f64(-mid) == (even | 0x8000)
        assert oracle.bf16_from_f64(math.nextafter(mid, 0.0)) == b
        assert oracle.bf16_from_f64(math.nextafter(mid, math.inf)) == b + 1


def test_bf16_rounds_directly_not_through_f32():
    # 1 + 2^-8 + 2^-30 lies just above the midpoint of 1 and 1 + 2^-7.  Rounding first to f32
    # (24 bits) lands exactly on the midpoint, which would then go to even (1.0): wrong.
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.bf16_from_f64(x) == 0x3F81
    assert oracle.bf16_from_f64(-x) == 0xBF81
    x = 1.0 + 3 * 2.0 ** -8 - 2.0 ** -30      # just below the midpoint of 0x3F81 and 0x3F82
    assert oracle.bf16_from_f64(x) == 0x3F81


def test_bf16_range_edges():
    big = oracle.bf16_to_f64(0x7F7F)
    assert big == (2 - 2.0 ** -7) * 2.0 ** 127
    assert oracle.bf16_from_f64(big) == 0x7F7F
    assert oracle.bf16_from_f64((2 - 2.0 ** -8) * 2.0 ** 127) == 0x7F80       # tie at the top: to even = inf
    assert oracle.bf16_from_f64(math.nextafter((2 - 2.0 ** -8) * 2.0 ** 127, 0)) == 0x7F7F
    assert oracle.bf16_from_f64(1e300) == 0x7F80 and oracle.bf16_from_f64(-1e300) == 0xFF80
    assert oracle.bf16_from_f64(math.inf) == 0x7F80
    assert oracle.bf16_from_f64(0.0) == 0 and oracle.bf16_from_f64(-0.0) == 0x8000
    tiny = 2.0 ** -133                       # smallest subnormal
    assert oracle.bf16_from_f64(tiny) == 1
    assert oracle.bf16_from_f64(tiny / 2) == 0          # tie to even (0)
    assert oracle.bf16_from_f64(tiny * 1.5) == 2        # tie to even (2)
    assert oracle.bf16_from_f64(tiny * 0.5000001) == 1
    assert oracle.bf16_from_f64(2.0 ** -126) == 0x0080  # smallest normal
    assert oracle.bf16_from_f64(1e-300) == 0
    assert oracle.bf16_from_f64(float("nan")) & 0x7FC0 == 0x7FC0


def test_bf16_matches_exact_rational_rounding_on_random_doubles():
    rng = np.random.Generator(np.random.PCG64(11))
    xs = np.concatenate([rng.standard_normal(4000), rng.standard_normal(2000) * 1e-38,
                         rng.standard_normal(2000) * 1e38, rng.standard_normal(2000) * 2.0 ** -130])
    for x in xs:
        assert oracle.bf16_from_f64(float(x)) == round_to_bf16_bits(float(x)), x


def test_f32_rounding_is_nearest_even():
    L = oracle.lib()
    one, nxt = 1.0, f32_of_bits(0x3F800001)
    mid = (one + nxt) / 2
    assert L.orc_f32_from_f64(mid) == one                    # tie to even mantissa
    assert L.orc_f32_from_f64(math.nextafter(mid, 2.0)) == nxt
    nxt2 = f32_of_bits(0x3F800002)
    assert L.orc_f32_from_f64((nxt + nxt2) / 2) == nxt2      # tie to even the other way
    assert L.orc_f32_from_f64(0.1) == np.float32(0.1)


def test_input_generator_bf16_codec_agrees():
    # the seeded generator's own float32 -> bf16 step must produce valid nearest-even patterns,
    # otherwise both sides would start from inputs that are not what the recipe says
    from pg_workloads import f32_to_bf16_bits, bf16_bits_to_f32
    rng = np.random.Generator(np.random.PCG64(3))
    x = rng.standard_normal(5000, dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    for xi, bi in zip(x[:2000], bits[:2000]):
        assert int(bi) == round_to_bf16_bits(float(xi))
    back = bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
