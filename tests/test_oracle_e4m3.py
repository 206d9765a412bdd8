"""Pins for the oracle's E4M3 encode/decode (Sec. 2.2 grid, Sec. 4.1 range) that do not use the
oracle as its own expected value: hand-written fixtures, exact rational brute force over all
codes, an independent library's cast, and ordering/tie invariants."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import w4a8_oracle as o

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_pairs(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _exact_value(code: int) -> Fraction:
    """E4M3 value of a code as an exact rational, from the bit fields (bias 7)."""
    s, e, m = code >> 7, (code >> 3) & 0xF, code & 7
    v = Fraction(m, 8) * Fraction(1, 64) if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
    return -v if s else v


FINITE = [c for c in range(256) if (c & 0x7F) != 0x7F]


def _brute_nearest(t: float) -> int:
    """Scan every finite code; nearest value, ties to the even code, sign taken from t."""
    ft = Fraction(t)
    best, best_d = None, None
    for c in range(0x7F):
        d = abs(abs(ft) - _exact_value(c))
        if best is None or d < best_d or (d == best_d and c % 2 == 0):
            best, best_d = c, d
    return best | (0x80 if np.signbit(np.float32(t)) else 0)


def test_landmarks_fixture():
    for byte, val in _read_pairs("e4m3_landmarks.txt"):
        b = int(byte, 16)
        got = o.e4m3_decode(np.array([b], dtype=np.uint8))[0]
        assert got == float(val) and np.signbit(got) == val.startswith("-")
        assert o.e4m3_encode(np.array([float(val)], dtype=np.float32))[0] == b


def test_int4_codes_fixture_is_exact():
    rows = _read_pairs("e4m3_int4_codes.txt")
    assert [int(r[0]) for r in rows] == list(range(-8, 8))
    q = np.array([int(r[0]) for r in rows], dtype=np.int8)
    want = np.array([int(r[1], 16) for r in rows], dtype=np.uint8)
    assert np.array_equal(o.dequant_codes_to_e4m3(q), want)
    # exactly representable: decoding gives the integer back (also for the unsigned range 0..15)
    assert np.array_equal(o.e4m3_decode(want), q.astype(np.float64))
    u = np.arange(0, 16)
    assert np.array_equal(o.e4m3_decode(o.e4m3_encode(u.astype(np.float32))), u.astype(np.float64))


def test_decode_matches_exact_bitfields():
    v = o.e4m3_decode(np.arange(256, dtype=np.uint8))
    for c in range(256):
        if (c & 0x7F) == 0x7F:
            assert np.isnan(v[c])
        else:
            assert Fraction(float(v[c])) == _exact_value(c)
    assert np.nanmax(v) == 448.0 and np.nanmin(v) == -448.0     # Sec. 4.1 range
    assert np.all(np.diff(v[:0x7F]) > 0)                          # monotone in the code


def test_roundtrip_all_codes():
    codes = np.array(FINITE, dtype=np.uint8)
    assert np.array_equal(o.e4m3_encode(o.e4m3_decode(codes).astype(np.float32)), codes)
    assert o.e4m3_encode(np.array([np.nan], dtype=np.float32))[0] == 0x7F
    assert np.isnan(o.e4m3_decode(np.array([0x7F, 0xFF], dtype=np.uint8))).all()


def test_midpoints_and_neighbours():
    """Every midpoint between adjacent grid points goes to the even code; one float32 step to
    either side goes to that side."""
    pts, want = [], []
    for c in range(0x7E):
        lo, hi = float(_exact_value(c)), float(_exact_value(c + 1))
        mid = np.float32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2                       # midpoints are float32-exact
        even = c if c % 2 == 0 else c + 1
        pts += [mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))]
        want += [even, c, c + 1]
    pts = np.array(pts, dtype=np.float32)
    want = np.array(want, dtype=np.uint8)
    assert np.array_equal(o.e4m3_encode(pts), want)
    assert np.array_equal(o.e4m3_encode(-pts), want | 0x80)


def test_underflow_overflow_and_specials():
    f = np.float32
    x = np.array([2.0 ** -10, np.nextafter(f(2.0 ** -10), f(1)), np.nextafter(f(2.0 ** -10), f(0)),
                  1e-30, 448, 463.9, 464, 465, 1e6, 3.4e38, np.inf, -np.inf, 0.0, -0.0, -1e-30],
                 dtype=np.float32)
    want = np.array([0x00, 0x01, 0x00, 0x00, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0x00, 0x80, 0x80],
                    dtype=np.uint8)
    assert np.array_equal(o.e4m3_encode(x), want)


def test_encode_against_exact_brute_force():
    rng = np.random.default_rng(7)
    x = np.concatenate([
        rng.standard_normal(600) * np.exp(rng.uniform(-8, 7, 600)),
        rng.uniform(-470, 470, 300), rng.uniform(-0.02, 0.02, 300)]).astype(np.float32)
    got = o.e4m3_encode(x)
    for t, g in zip(x, got):
        assert g == _brute_nearest(float(t)), (t, hex(g))


def test_encode_against_independent_library():
    """torch's CPU float8_e4m3fn cast is an independent implementation of the same grid with
    round-half-even; it overflows to NaN above 464 where the method saturates, so compare inside."""
    rng = np.random.default_rng(11)
    x = np.concatenate([
        rng.standard_normal(400000) * np.exp(rng.uniform(-12, 6, 400000)),
        rng.uniform(-464, 464, 200000),
        np.arange(-464, 464, 0.0625)]).astype(np.float32)
    x = x[np.abs(x) <= 464]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(o.e4m3_encode(x), want)
    # and every bf16-representable float32 in range (all 2^16 patterns)
    allbf = (np.arange(1 << 16, dtype=np.uint32) << 16).view(np.float32)
    keep = np.isfinite(allbf) & (np.abs(allbf) <= 464)
    want = torch.from_numpy(allbf[keep]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(o.e4m3_encode(allbf[keep]), want)


def test_bf16_rounding_helper():
    """round_to_bf16_bits is a single correct rounding: exact rational check on random values,
    identity on bf16 values, ties to even."""
    rng = np.random.default_rng(3)
    y = rng.standard_normal(300) * np.exp(rng.uniform(-60, 60, 300))
    bits = o.round_to_bf16_bits(y)
    val = o.bf16_bits_to_f32(bits).astype(np.float64)
    for yi, vi, bi in zip(y, val, bits):
        up = o.bf16_bits_to_f32(np.array([bi + 1], dtype=np.uint16))[0]
        dn = o.bf16_bits_to_f32(np.array([bi - 1], dtype=np.uint16))[0]
        d = abs(Fraction(float(vi)) - Fraction(float(yi)))
        assert d <= abs(Fraction(float(up)) - Fraction(float(yi)))
        assert d <= abs(Fraction(float(dn)) - Fraction(float(yi)))
        assert d <= Fraction(float(o.bf16_half_ulp(yi)))
    allb = np.arange(1 << 16, dtype=np.uint16)
    f = o.bf16_bits_to_f32(allb)
    fin = np.isfinite(f)
    assert np.array_equal(o.round_to_bf16_bits(f[fin].astype(np.float64)), allb[fin])
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: goes to the even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert o.round_to_bf16_bits(np.array([1 + 2.0 ** -8]))[0] == 0x3F80
    assert o.round_to_bf16_bits(np.array([1 + 3 * 2.0 ** -8]))[0] == 0x3F82


def test_bf16_half_ulp_exact_values():
    """bf16_half_ulp pinned from both sides (a value twice or half as large fails): hand values at the ends of a binade,
    in the subnormal range, and for every finite bf16 pattern exactly half the distance to the next pattern away from
    zero (bf16 has 8 significant bits: spacing 2^(e-7) in [2^e, 2^(e+1)), 2^-133 below 2^-126)."""
    assert o.bf16_half_ulp(1.0) == 2.0 ** -8
    assert o.bf16_half_ulp(np.nextafter(2.0, 0.0)) == 2.0 ** -8            # still the binade of 1.0
    assert o.bf16_half_ulp(2.0) == 2.0 ** -7
    assert o.bf16_half_ulp(-3.0) == 2.0 ** -7
    assert o.bf16_half_ulp(448.0) == 2.0 ** 0                                # 448 = 1.75 * 2^8: spacing 2, half of it 1
    assert o.bf16_half_ulp(2.0 ** -126) == 2.0 ** -134                      # smallest normal
    assert o.bf16_half_ulp(2.0 ** -130) == 2.0 ** -134 and o.bf16_half_ulp(0.0) == 2.0 ** -134   # subnormals: fixed spacing 2^-133
    bits = np.arange(0x7F7F, dtype=np.uint16)                                # 0 .. the pattern before the largest finite one
    x = o.bf16_bits_to_f32(bits).astype(np.float64)
    nxt = o.bf16_bits_to_f32(bits + np.uint16(1)).astype(np.float64)
    assert np.array_equal(o.bf16_half_ulp(x), (nxt - x) / 2)
    assert np.array_equal(o.bf16_half_ulp(-x), (nxt - x) / 2)
    # strictly inside a binade the value does not change; it doubles exactly at a power of two
    assert o.bf16_half_ulp(1.9999) == o.bf16_half_ulp(1.0001) == 2.0 ** -8
