"""Pins for the oracle's activation quantizer (Eq. 13), the symmetric INT4 round-to-nearest
quantizer (Eq. 1, symmetric case) and the two storage formats."""
from fractions import Fraction

import numpy as np

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import synthetic as syn

FINITE = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)


def test_quantize_act_idempotent_on_grid_with_pow2_scale():
    for s in (1.0, 0.25, 8.0, 2.0 ** -20):
        x = (o.e4m3_decode(FINITE) * s).astype(np.float32)
        assert np.array_equal(o.quantize_act(x, np.float32(s)), FINITE)


def test_quantize_act_pow2_scale_invariance_and_amax():
    rng = np.random.default_rng(5)
    x = syn.make_activations(rng, 16, 512, 0.01, 20.0)
    s = o.act_scale_from_amax(x)
    a = o.quantize_act(x, s)
    assert np.array_equal(o.quantize_act(x * np.float32(4), s * np.float32(4)), a)
    i = np.unravel_index(np.argmax(np.abs(x)), x.shape)
    assert a[i] & 0x7F == 0x7E                                   # the amax element lands on +-448
    assert s == syn.static_act_scale(x)                          # workload recipe == Eq. 13 rule
    assert Fraction(float(s)) == Fraction(float(np.float32(np.abs(x).max()) / np.float32(448)))


def test_quantize_act_is_nearest_grid_point_of_fp32_quotient():
    """Definition check with exact rationals on a small sample: the code is the grid point nearest
    to the float32 quotient x / s."""
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(200) * 3).astype(np.float32)
    s = np.float32(0.0123)
    got = o.e4m3_decode(o.quantize_act(x, s))
    grid = o.e4m3_decode(FINITE)
    for xi, gi in zip(x, got):
        quo = Fraction(float(np.float32(xi / s)))
        best = min(abs(quo - Fraction(float(v))) for v in grid)
        assert abs(quo - Fraction(float(gi))) == best


def test_quantize_act_bf16_input_and_saturation():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x7F80, 0xFF80, 0x7FC0, 0x0000, 0x8000], dtype=np.uint16)
    got = o.quantize_act(bits, np.float32(1.0), x_is_bf16_bits=True)
    assert list(got) == [0x38, 0xB8, 0x40, 0x7E, 0xFE, 0x7F, 0x00, 0x80]
    # a static scale that is too small for the data: saturate to +-448, never NaN
    assert list(o.quantize_act(np.array([1000.0, -1000.0], np.float32), np.float32(1.0))) == [0x7E, 0xFE]


def test_rtn_hand_cases_and_ties():
    # one group of 8 with amax 7 -> s = 1: codes are the half-even roundings; nothing reaches -8
    w = np.array([[7.0, -7.0, 0.5, 1.5, 2.5, -0.5, -1.5, 3.49]], dtype=np.float32)
    q, s = o.rtn_quantize_weights(w, 8)
    assert s.tolist() == [[1.0]] and q.tolist() == [[7, -7, 0, 2, 2, 0, -2, 3]]
    # all-zero group: scale 1, codes 0
    q, s = o.rtn_quantize_weights(np.zeros((2, 64), np.float32), 32)
    assert np.all(s == 1.0) and not q.any()


def test_rtn_roundtrip_pow2_scales():
    rng = np.random.default_rng(8)
    q0 = rng.integers(-7, 8, size=(32, 256)).astype(np.int8)
    q0[:, ::32] = 7                                              # every group of 32 holds a 7
    s0 = np.ldexp(1.0, rng.integers(-12, 3, size=(32, 8))).astype(np.float32)
    w = (q0.reshape(32, 8, 32) * s0[:, :, None]).reshape(32, 256).astype(np.float32)
    q, s = o.rtn_quantize_weights(w, 32)
    assert np.array_equal(q, q0) and np.array_equal(s, s0)


def test_rtn_reconstruction_error_bound():
    """|W - q*s| <= s/2 for every weight (round-to-nearest), and codes stay in [-7, 7] for
    absmax/7 scales."""
    w = syn.make_weights(np.random.default_rng(9), 64, 512)
    q, s = o.rtn_quantize_weights(w, 128)
    rec = q.reshape(64, 4, 128) * s[:, :, None].astype(np.float64)
    err = np.abs(rec.reshape(64, 512) - w)
    assert np.all(err <= np.repeat(s, 128, axis=1) * 0.5 * (1 + 1e-6))
    assert q.min() >= -7 and q.max() <= 7
    assert np.all(np.abs(q).reshape(64, 4, 128).max(axis=2) == 7)


def test_canonical_pack_hand_row_and_all_bytes():
    q = np.array([[1, -1, -8, 7]], dtype=np.int8)
    assert o.pack_canonical(q).tolist() == [[0xF1, 0x78]]       # low nibble first
    # all 256 byte values survive unpack -> pack
    allb = np.arange(256, dtype=np.uint8).reshape(1, 256)
    assert np.array_equal(o.pack_canonical(o.unpack_canonical(allb)), allb)
    u = o.unpack_canonical(allb)
    assert u.min() == -8 and u.max() == 7


def test_tiled_pack_is_a_permutation_with_the_documented_positions():
    rng = np.random.default_rng(10)
    n, k = 40, 384                                               # ragged N: pads to 48
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    buf = o.pack_tiled(q)
    assert buf.size == 48 * k // 2
    assert np.array_equal(o.unpack_tiled(buf, n, k), q)
    assert np.array_equal(buf, o.pack_tiled_by_offsets(q))          # reshape form == explicit offsets
    # hand-computed positions and nibble patterns, straight from the layout's definition
    hand = {0: 0x0, 1: 0x1, 2: 0x2, 3: 0x3, 4: 0x4, 5: 0x5, 6: 0x6, 7: 0x7,
            -1: 0x9, -2: 0xA, -3: 0xB, -4: 0xC, -5: 0xD, -6: 0xE, -7: 0xF, -8: 0x8}      # sign-magnitude; -8 = 1000
    def at(nn, kk):
        t, i, c, kq, p = nn // 16, nn % 16, kk // 128, (kk % 128) // 32, kk % 32
        byte = (t * (k // 128) + c) * 1024 + (16 * kq + i) * 16 + 4 * (p // 8) + (p % 8) % 4
        return int(buf[byte]) >> 4 if (p % 8) >= 4 else int(buf[byte]) & 0xF
    for nn, kk in [(0, 0), (0, 4), (0, 7), (0, 8), (1, 0), (15, 31), (16, 32), (17, 127), (39, 383), (5, 200)]:
        assert at(nn, kk) == hand[int(q[nn, kk])]
    assert [int(v) for v in o.tiled_nibble(np.arange(-8, 8))] == [hand[c] for c in range(-8, 8)]
    assert np.array_equal(o.tiled_nibble_to_code(np.arange(16)), [0, 1, 2, 3, 4, 5, 6, 7, -8, -1, -2, -3, -4, -5, -6, -7])
    # one code set, everything else zero: exactly one nibble of the buffer is non-zero
    z = np.zeros((16, 128), np.int8)
    z[3, 37] = -3                                                # kq=1, p=5 -> d=0, e=5 -> byte 1, high nibble
    b = o.pack_tiled(z)
    assert np.flatnonzero(b).tolist() == [(16 * 1 + 3) * 16 + 1] and b[(16 + 3) * 16 + 1] == 0xB0
    z[3, 37] = -8
    assert o.pack_tiled(z)[(16 + 3) * 16 + 1] == 0x80
    # padding rows are code 0
    assert not o.unpack_tiled(buf, 48, k)[40:].any()


def test_scale_tiling_roundtrip_and_position():
    s = np.arange(40 * 3, dtype=np.float32).reshape(40, 3) + 1
    t = o.tile_scales(s)
    assert t.size == 48 * 3
    assert np.array_equal(o.untile_scales(t, 40, 3), s)
    assert t[((17 // 16) * 3 + 2) * 16 + 17 % 16] == s[17, 2]
    assert not t.reshape(3, 3, 16)[2, :, 8:].any()              # rows 40..47 are padding


def test_scale_sign_marks_exactly_the_groups_that_hold_minus_eight():
    rng = np.random.default_rng(12)
    n, k, g = 40, 512, 128
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)        # no -8 anywhere ...
    s = rng.uniform(0.0, 1.0, size=(n, k // g)).astype(np.float32)
    s[5, 1] = 0.0
    assert not np.signbit(o.tile_scales(s, q)).any()
    assert np.array_equal(o.tile_scales(s, q), o.tile_scales(s))
    q[3, 130] = -8                                               # ... then in row 3 group 1, row 5 group 1 (zero scale), row 39 group 3
    q[5, 255] = -8
    q[39, 384] = -8
    t = o.tile_scales(s, q)
    mag, marks = o.untile_scales(t, n, k // g, with_marks=True)
    assert np.array_equal(mag, s)
    want = np.zeros((n, k // g), bool)
    want[3, 1] = want[5, 1] = want[39, 3] = True
    assert np.array_equal(marks, want)
    assert np.signbit(t[((3 // 16) * 4 + 1) * 16 + 3]) and t[((3 // 16) * 4 + 1) * 16 + 3] == -s[3, 1]
    # the mark is a hint only: the packed codes alone decode to the same integers
    assert np.array_equal(o.unpack_tiled(o.pack_tiled(q), n, k), q)


def test_pow2_quantizer_hand_example_and_invariants():
    """max|W| / 7 = 0.3 / 7 = 0.0428.. lies between 2^-5 and 2^-4: s = 2^-4; max|W| = 7 * 2^-3 exactly: s = 2^-3."""
    w = np.array([[0.3, -0.1, 0.05, 0.0, 0.875, -0.875, 0.25, 0.1]], dtype=np.float32)
    q, s = o.rtn_quantize_weights_pow2(w, 4)
    assert s.tolist() == [[2.0 ** -4, 2.0 ** -3]]
    assert q.tolist() == [[5, -2, 1, 0, 7, -7, 2, 1]]            # 0.3*16 = 4.8, 0.1*16 = 1.6, 0.05*16 = 0.8; 0.1*8 = 0.8
    rng = np.random.default_rng(31)
    w = syn.make_weights(rng, 48, 1024)
    w[0, :128] = 0.0
    q, s = o.rtn_quantize_weights_pow2(w, 128)
    mant, _ = np.frexp(s)
    assert np.all(mant == 0.5) and s[0, 0] == 1.0                # powers of two
    amax = np.abs(w.reshape(48, 8, 128)).max(axis=2).astype(np.float64)
    nz = amax > 0
    assert np.all(7.0 * s[nz] >= amax[nz] * (1 - 1e-7)) and np.all(7.0 * s[nz] < 2.0 * amax[nz] * (1 + 1e-7))
    assert q.min() >= -7 and q.max() <= 7
    rec = q.reshape(48, 8, 128) * s[..., None].astype(np.float64)
    assert np.all(np.abs(rec - w.reshape(48, 8, 128)) <= 0.5 * s[..., None])
    # with a power-of-two scale the quotient is exact, so the code is the nearest integer of the exact quotient
    exact = w.reshape(48, 8, 128).astype(np.float64) / s[..., None]
    assert np.array_equal(q.reshape(48, 8, 128), np.rint(exact).astype(np.int8))
