"""Pins for the oracle's asymmetric format: unsigned 4-bit codes with per-group scale and zero-point
(Eq. 1 in its asymmetric form, Eq. 8-9, Eq. 14), its E4M3 operand bytes and its storage."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import synthetic as syn


def test_quantizer_hand_example():
    """Two groups of four weights on a grid where every step of Eq. 1 is exact in binary:
    lo = -1, hi = 2.75, s = 3.75 / 15 = 0.25, z = round(1 / 0.25) = 4, u = round(W / 0.25 + 4)."""
    w = np.array([[-1.0, 0.25, 1.5, 2.75, -1.0, 0.3, 0.9, 2.75]], dtype=np.float32)
    u, s, z = o.asym_quantize_weights(w, 4)
    assert s.tolist() == [[0.25, 0.25]] and z.tolist() == [[4, 4]]
    # 0.3 / 0.25 + 4 = 5.2 -> 5;  0.9 / 0.25 + 4 = 7.6 -> 8
    assert u.tolist() == [[0, 5, 10, 15, 0, 5, 8, 15]]


def test_quantizer_one_signed_and_zero_groups():
    """The range is extended to contain zero: an all-positive group gets z = 0, an all-negative one z = 15,
    an all-zero one s = 1, z = 0, codes 0."""
    w = np.array([[1.0, 2.0, 3.0, 7.5, -7.5, -1.0, -2.0, -3.0, 0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    u, s, z = o.asym_quantize_weights(w, 4)
    assert s.tolist() == [[0.5, 0.5, 1.0]] and z.tolist() == [[0, 15, 0]]
    assert u.tolist() == [[2, 4, 6, 15, 0, 13, 11, 9, 0, 0, 0, 0]]


def test_quantizer_picks_the_nearest_level_exact_rationals():
    """Definition check, independent of the round(W/s + z) formula: with the oracle's own s and z, every code is
    the level u in 0..15 whose value (u - z) s is nearest to the weight, in exact rational arithmetic (weights whose
    two best levels are within 1e-4 s of a tie are left out: there the float32 evaluation order decides)."""
    rng = np.random.default_rng(11)
    w = syn.make_weights(rng, 6, 256)
    u, s, z = o.asym_quantize_weights(w, 128)
    checked = 0
    for n in range(6):
        for k in range(256):
            g = k // 128
            sf, zf, wf = Fraction(float(s[n, g])), int(z[n, g]), Fraction(float(w[n, k]))
            dist = sorted((abs(wf - (lv - zf) * sf), lv) for lv in range(16))
            if dist[1][0] - dist[0][0] < sf / 10000:
                continue
            assert dist[0][1] == int(u[n, k])
            checked += 1
    assert checked > 1500


def test_quantizer_invariants_on_llama_shaped_weights():
    rng = np.random.default_rng(12)
    w = syn.make_weights(rng, 64, 1024)
    u, s, z = o.asym_quantize_weights(w, 128)
    assert u.dtype == np.uint8 and u.max() <= 15 and z.max() <= 15 and np.all(s > 0)
    ug = u.reshape(64, 8, 128)
    wg = w.reshape(64, 8, 128)
    # both ends of the range are used: the smallest weight of a group takes code 0, the largest code 15
    assert np.all(np.take_along_axis(ug, wg.argmin(axis=2)[..., None], axis=2) == 0)
    assert np.all(np.take_along_axis(ug, wg.argmax(axis=2)[..., None], axis=2) == 15)
    # Eq. 2: the reconstruction (u - z) s is within half a step of the weight (plus float32 rounding of W/s + z)
    rec = (ug.astype(np.float64) - z[..., None]) * s[..., None].astype(np.float64)
    assert np.all(np.abs(rec - wg) <= 0.5 * s[..., None] * (1 + 1e-5))
    # Eq. 8: fifteen steps span max - min of a group that straddles zero
    span = wg.max(axis=2).astype(np.float64) - wg.min(axis=2)
    assert np.allclose(15.0 * s, span, rtol=1e-6)


def test_operand_bytes_are_the_exact_integers():
    """Every (code, zero-point) pair: the byte decodes to code - zero_point exactly, and equals an independent
    library's E4M3 cast of that integer."""
    import torch
    uu, zz = np.meshgrid(np.arange(16, dtype=np.uint8), np.arange(16, dtype=np.uint8), indexing="ij")
    u = uu.reshape(256, 1)
    z = zz.reshape(256, 1)
    b = o.dequant_asym_to_e4m3(u, z, 1)
    assert np.array_equal(o.e4m3_decode(b)[:, 0], u[:, 0].astype(np.float64) - z[:, 0])
    ref = torch.tensor((u.astype(np.float32) - z.astype(np.float32))[:, 0]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(b[:, 0] & 0x7F, ref & 0x7F)            # magnitudes; zero has no sign to compare
    assert np.array_equal(b[:, 0][u[:, 0] != z[:, 0]], ref[u[:, 0] != z[:, 0]])


def test_zero_point_belongs_to_its_group():
    """A wrong group index for z shows here: different zero-points per group, codes chosen so that the integers
    are known by construction."""
    u = np.array([[3, 3, 9, 9, 15, 0]], dtype=np.uint8)
    z = np.array([[1, 10, 7]], dtype=np.uint8)
    d = o.e4m3_decode(o.dequant_asym_to_e4m3(u, z, 2))
    assert d.tolist() == [[2, 2, -1, -1, 8, -7]]


def _tiny_case(seed, m, k, n, g):
    rng = np.random.default_rng(seed)
    x8 = rng.choice(np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8), size=(m, k))
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, k // g), dtype=np.uint8)
    s = (rng.random((n, k // g), dtype=np.float32) + np.float32(0.5)) * np.float32(0.01)
    return x8, u, z, s


def test_linear_asym_brute_force_exact_rationals():
    x8, u, z, s = _tiny_case(21, 2, 8, 3, 4)
    sx = np.float32(0.37)
    y, a = o.linear_ref_asym(x8, sx, u, z, s, 4)
    xd = o.e4m3_decode(x8)
    for m in range(2):
        for n in range(3):
            tot = Fraction(0)
            tot_abs = Fraction(0)
            for k in range(8):
                term = Fraction(float(xd[m, k])) * (int(u[n, k]) - int(z[n, k // 4])) * Fraction(float(s[n, k // 4]))
                tot += term
                tot_abs += abs(term)
            assert abs(Fraction(float(y[m, n])) - tot * Fraction(float(sx))) <= abs(tot) * Fraction(1, 10 ** 12) + Fraction(1, 10 ** 300)
            assert abs(Fraction(float(a[m, n])) - tot_abs * Fraction(float(sx))) <= tot_abs * Fraction(1, 10 ** 12)


def test_linear_asym_equals_dense_product_with_eq14_weights():
    """Eq. 14 written out: W_hat[n, k] = (u - z) s built entry by entry, then one dense float64 product."""
    x8, u, z, s = _tiny_case(22, 5, 256, 7, 128)
    sx = np.float32(0.02)
    w_hat = np.zeros((7, 256))
    for n in range(7):
        for k in range(256):
            w_hat[n, k] = (int(u[n, k]) - int(z[n, k // 128])) * float(s[n, k // 128])
    ref = float(sx) * (o.e4m3_decode(x8) @ w_hat.T)
    y, a = o.linear_ref_asym(x8, sx, u, z, s, 128)
    assert np.allclose(y, ref, rtol=0, atol=1e-12 * a.max())


def test_linear_asym_reduces_to_the_symmetric_layer():
    """Codes q + 8 with zero-point 8 are the signed codes q: the two layers agree to the last bit."""
    rng = np.random.default_rng(23)
    x8, _, _, s = _tiny_case(23, 4, 256, 9, 128)
    q = rng.integers(-8, 8, size=(9, 256)).astype(np.int8)
    u = (q.astype(np.int16) + 8).astype(np.uint8)
    z = np.full((9, 2), 8, dtype=np.uint8)
    y0, a0 = o.linear_ref(x8, np.float32(0.1), q, s, 128)
    y1, a1 = o.linear_ref_asym(x8, np.float32(0.1), u, z, s, 128)
    assert np.array_equal(y0, y1) and np.array_equal(a0, a1)


def test_asym_storage_by_explicit_offsets():
    rng = np.random.default_rng(24)
    n, k, g = 37, 384, 128
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, k // g), dtype=np.uint8)
    s = rng.random((n, k // g), dtype=np.float32)
    packed = o.pack_tiled_asym(u)
    params = o.tile_params_asym(s, z)
    n_pad, ng = 48, k // g
    assert packed.size == n_pad * k // 2 and params.size == (n_pad // 16) * ng * 80
    # nibbles: the positions the tiled format defines; the nibble spelled out from its definition: the code is
    # 7.5 + h, h = +-(m + 0.5); codes 8..15 are 0mmm with m = code - 8, codes 0..7 are 1mmm with m = 7 - code
    patterns = {8: 0b0000, 9: 0b0001, 10: 0b0010, 11: 0b0011, 12: 0b0100, 13: 0b0101, 14: 0b0110, 15: 0b0111,
                7: 0b1000, 6: 0b1001, 5: 0b1010, 4: 0b1011, 3: 0b1100, 2: 0b1101, 1: 0b1110, 0: 0b1111}
    for code, pat in patterns.items():
        h = (-1 if pat & 8 else 1) * ((pat & 7) + 0.5)
        assert 7.5 + h == code
    byte, nib = o._tiled_destination(n_pad, k)
    want = np.zeros(n_pad * k // 2, dtype=np.uint8)
    for nn in range(n_pad):
        for kk in range(k):
            code = int(u[nn, kk]) if nn < n else 0
            want[byte[nn, kk]] |= patterns[code] << (4 * int(nib[nn, kk]))
    assert np.array_equal(packed, want)
    # records: scale (n, g) as little-endian float32 at ((n // 16) * ng + g) * 80 + 4 * (n % 16), zero-point
    # at ((n // 16) * ng + g) * 80 + 64 + n % 16
    for nn in range(n_pad):
        for gg in range(ng):
            base = ((nn // 16) * ng + gg) * 80
            sv = params[base + 4 * (nn % 16): base + 4 * (nn % 16) + 4].view("<f4")[0]
            zv = params[base + 64 + nn % 16]
            assert sv == (s[nn, gg] if nn < n else 0.0) and zv == (z[nn, gg] if nn < n else 0)
    assert np.array_equal(o.unpack_tiled_asym(packed, n, k), u)
    s2, z2 = o.untile_params_asym(params, n, ng)
    assert np.array_equal(s2, s) and np.array_equal(z2, z)


@pytest.mark.parametrize("g", [128, 256])
def test_quantize_then_layer_close_to_unquantized(g):
    """End to end on Llama-shaped synthetic weights: the layer on asymmetric 4-bit weights stays within the
    error the format implies (each weight off by at most s/2) of the layer on the unquantized weights."""
    rng = np.random.default_rng(25)
    w = syn.make_weights(rng, 32, 512)
    x = syn.make_activations(rng, 8, 512, 0.01, 20.0)
    sx = syn.static_act_scale(x)
    x8 = o.quantize_act(x, sx)
    u, s, z = o.asym_quantize_weights(w, g)
    y, _ = o.linear_ref_asym(x8, sx, u, z, s, g)
    xd = o.e4m3_decode(x8) * float(sx)
    ref = xd @ w.astype(np.float64).T
    bound = np.abs(xd) @ np.repeat(0.5 * s.astype(np.float64) * (1 + 1e-5), g, axis=1).T
    assert np.all(np.abs(y - ref) <= bound + 1e-12)


def test_literal_asym_bytes_hand_values_and_special_cases():
    """(u - z) * s8 on hand-picked cases: exact grid points, a tie (2^-10 * 3 / ... is covered by the E4M3 pins; here
    17 * 1 = 17 lies between 16 and 18 -> ties to the even mantissa, 16), saturation, zero."""
    u = np.array([[15, 0, 9, 7, 15, 15]], dtype=np.uint8)
    z = np.array([[7, 7, 7, 7, 0, 0]], dtype=np.uint8)             # groups of one weight
    s8 = np.array([[2.0, 3.0, 8.5, 100.0, 1.0, 40.0]], dtype=np.float32)
    _, w8 = o.linear_ref_asym_paper_literal(np.zeros((1, 6), np.uint8), np.float32(1), u, z, s8, np.ones(1), 1)
    # 8*2 = 16; -7*3 = -21 -> between -20 and -22: tie -> even mantissa: -20 (1.010 x 16) vs -22 (1.011 x 16) -> -20;
    # 2*8.5 = 17 -> tie between 16 and 18 -> 16; 0*100 = 0; 15*1 = 15; 15*40 = 600 -> 448
    assert o.e4m3_decode(w8).tolist() == [[16.0, -20.0, 16.0, 0.0, 15.0, 448.0]]


def test_literal_asym_reduces_to_known_layers():
    rng = np.random.default_rng(26)
    x8, u, z, _ = _tiny_case(26, 4, 256, 9, 128)
    # power-of-two scales keep (u - z) * s8 on the grid: the literal layer equals the factored one (Eq. 14)
    e = rng.integers(-3, 3, size=(9, 2))
    s8 = np.ldexp(1.0, e).astype(np.float32)
    s_out = (rng.random(9) + 0.5).astype(np.float32)
    y_lit, w8 = o.linear_ref_asym_paper_literal(x8, np.float32(0.1), u, z, s8, s_out, 128)
    y_fac, _ = o.linear_ref_asym(x8, np.float32(0.1), u, z, s8, 128)
    assert np.allclose(y_lit, y_fac * s_out.astype(np.float64)[None, :], rtol=1e-13, atol=0)
    # zero-point 8 and codes q + 8: the signed two-level layer, byte for byte
    q = rng.integers(-8, 8, size=(9, 256)).astype(np.int8)
    s8r = (rng.random((9, 2), dtype=np.float32) + np.float32(0.2)) * np.float32(9.0)
    y0, b0 = o.linear_ref_paper_literal(x8, np.float32(0.1), q, s8r, s_out, 128)
    y1, b1 = o.linear_ref_asym_paper_literal(x8, np.float32(0.1), (q.astype(np.int16) + 8).astype(np.uint8),
                                             np.full((9, 2), 8, np.uint8), s8r, s_out, 128)
    assert np.array_equal(b0 & 0x7F, b1 & 0x7F) and np.array_equal(y0, y1)     # -0 / +0 bytes may differ in sign only
