"""Pins for the oracle's layer output (Eq. 10, 4, 11): hand loops, closed forms, an exact integer
special case, linearity, a library matmul on explicitly dequantized operands, and the
paper-literal reading collapsing onto the code-exact one for power-of-two scales."""
from fractions import Fraction

import numpy as np

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import synthetic as syn


def _case(seed, m, k, n, g):
    rng = np.random.default_rng(seed)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    q, s_w = o.rtn_quantize_weights(w, g)
    return o.quantize_act(x, s_x), s_x, q, s_w


def test_hand_loops_with_exact_rationals():
    x8, s_x, q, s_w = _case(1, 3, 256, 4, 128)
    y, a = o.linear_ref(x8, s_x, q, s_w, 128)
    xd = o.e4m3_decode(x8)
    for m in range(3):
        for n in range(4):
            tot, tot_abs = Fraction(0), Fraction(0)
            for k in range(256):
                term = Fraction(float(xd[m, k])) * int(q[n, k]) * Fraction(float(s_w[n, k // 128]))
                tot += term
                tot_abs += abs(term)
            tot *= Fraction(float(s_x))
            tot_abs *= Fraction(float(s_x))
            assert abs(Fraction(float(y[m, n])) - tot) <= abs(tot_abs) * Fraction(1, 10 ** 13)
            assert abs(Fraction(float(a[m, n])) - tot_abs) <= tot_abs * Fraction(1, 10 ** 13)


def test_one_hot_rows_closed_form():
    k, g = 512, 128
    q = np.zeros((5, k), np.int8)
    hot = [0, 127, 128, 300, 511]
    val = [7, -8, 1, -3, 5]
    for r, (kk, v) in enumerate(zip(hot, val)):
        q[r, kk] = v
    s_w = (np.arange(5 * 4, dtype=np.float32).reshape(5, 4) + 1) / 64
    x8 = np.random.default_rng(2).integers(0, 0x7F, size=(2, k)).astype(np.uint8)
    y, _ = o.linear_ref(x8, np.float32(0.5), q, s_w, g)
    xd = o.e4m3_decode(x8)
    for r, (kk, v) in enumerate(zip(hot, val)):
        assert np.array_equal(y[:, r], 0.5 * float(s_w[r, kk // g]) * xd[:, kk] * v)


def test_exact_integer_case_matches_int64_matmul():
    rng = np.random.default_rng(3)
    m, k, n, g = 4, 1024, 24, 128
    xi = rng.integers(-8, 9, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    e = rng.integers(-3, 4, size=(n, k // g))
    s_w = np.ldexp(1.0, e).astype(np.float32)
    y, _ = o.linear_ref(x8, np.float32(2.0), q, s_w, g)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, k // g, g).astype(np.int64),
                     q.reshape(n, k // g, g).astype(np.int64))            # exact integers
    want = 2.0 * (part * np.ldexp(1.0, e)[None]).sum(axis=2)
    assert np.array_equal(y, want)


def test_library_matmul_on_dequantized_operands():
    """Plain Y = X_hat . W_hat^T with W_hat = q * s (Eq. 10, z = 0) materialised: the factored form
    used by linear_ref is the same number up to float64 rounding."""
    x8, s_x, q, s_w = _case(4, 8, 1024, 64, 128)
    y, a = o.linear_ref(x8, s_x, q, s_w, 128)
    w_hat = q.astype(np.float64) * np.repeat(s_w.astype(np.float64), 128, axis=1)
    x_hat = o.e4m3_decode(x8) * float(s_x)
    want = x_hat @ w_hat.T
    assert np.max(np.abs(y - want)) <= 1e-12 * np.max(a)
    # per-output-channel scales are the group_size = K case
    qc, sc = o.rtn_quantize_weights(syn.make_weights(np.random.default_rng(4), 64, 1024), 1024)
    yc, _ = o.linear_ref(x8, s_x, qc, sc, 1024)
    assert np.allclose(yc, (x_hat @ qc.T.astype(np.float64)) * sc[:, 0][None, :], rtol=1e-12, atol=0)


def test_linearity_in_scales():
    x8, s_x, q, s_w = _case(5, 4, 512, 16, 128)
    y, _ = o.linear_ref(x8, s_x, q, s_w, 128)
    y2, _ = o.linear_ref(x8, np.float32(2) * s_x, q, s_w, 128)
    assert np.array_equal(y2, 2 * y)
    s2 = s_w.copy()
    s2[:, 1] *= 2
    y3, _ = o.linear_ref(x8, s_x, q, s2, 128)
    only_g1, _ = o.linear_ref(x8[:, 128:256], s_x, q[:, 128:256], s_w[:, 1:2], 128)
    assert np.allclose(y3 - y, only_g1, rtol=1e-9, atol=1e-12 * np.abs(y).max())


def test_tolerance_rule():
    ref = np.array([[1.0, 0.0, -2.0]])
    a = np.array([[10.0, 10.0, 10.0]])
    assert o.within_tolerance(ref * (1 + 1.9e-3), ref, a)[0]
    assert not o.within_tolerance(ref * (1 + 2.1e-3), ref, a)[0]
    assert o.within_tolerance(np.array([[1.0, 3.0e-4, -2.0]]), ref, a)[0]      # floor = 2e-3 * 2^-6 * A = 3.125e-4
    assert not o.within_tolerance(np.array([[1.0, 3.2e-4, -2.0]]), ref, a)[0]


def test_paper_literal_mode():
    rng = np.random.default_rng(6)
    n, k, g = 16, 256, 128
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    x8 = rng.integers(0, 0x7F, size=(3, k)).astype(np.uint8)
    # power-of-two FP8-domain scales: products are exact on the grid, so the two readings agree
    s8 = np.ldexp(1.0, rng.integers(-2, 4, size=(n, k // g))).astype(np.float32)
    s_out = (rng.uniform(0.5, 2, n)).astype(np.float32)
    y_lit, w8 = o.linear_ref_paper_literal(x8, np.float32(0.25), q, s8, s_out, g)
    y_code, _ = o.linear_ref(x8, np.float32(0.25), q, s8 * s_out[:, None], g)
    assert np.allclose(y_lit, y_code, rtol=1e-12, atol=0)
    assert np.array_equal(o.e4m3_decode(w8), q * np.repeat(s8, g, axis=1).astype(np.float64))
    # general scales: each weight is the nearest grid point of the float32 product (<= 2^-4 relative)
    s8 = rng.uniform(1.0, 50.0, size=(n, k // g)).astype(np.float32)
    _, w8 = o.linear_ref_paper_literal(x8, np.float32(1), q, s8, s_out, g)
    prod = q.astype(np.float32) * np.repeat(s8, g, axis=1)
    assert np.array_equal(w8, o.e4m3_encode(np.clip(prod, -448, 448)))
    nz = prod != 0
    assert np.all(np.abs(o.e4m3_decode(w8)[nz] - prod[nz]) <= np.abs(prod[nz]) * 2.0 ** -4)


def test_block_ref_wiring_small():
    """Tiny block: each stage of block_ref equals quantize -> linear_ref -> bf16 on the previous
    stage's bf16 tensor; O reads the first `hidden` columns of QKV; SiLU*mul closed form."""
    rng = np.random.default_rng(12)
    hidden, ffn, g, m = 256, 384, 128, 3
    dims = {"qkv": (hidden, hidden + 128), "o": (hidden, hidden), "gate_up": (hidden, 2 * ffn), "down": (ffn, hidden)}
    layers = {nm: o.rtn_quantize_weights(syn.make_weights(rng, n, k, 0.05), g) for nm, (k, n) in dims.items()}
    x = syn.f32_to_bf16_bits(syn.make_activations(rng, m, hidden, 0.01, 20.0))
    sx = {"qkv": np.float32(0.05), "o": np.float32(0.01), "gate_up": np.float32(0.004), "down": np.float32(1e-4)}
    out = o.block_ref(x, layers, sx, g, hidden, ffn)
    x8 = o.quantize_act(np.ascontiguousarray(out["qkv"][:, :hidden]), sx["o"], x_is_bf16_bits=True)
    assert np.array_equal(x8, out["o_x8"])
    y, _ = o.linear_ref(x8, sx["o"], *layers["o"], g)
    assert np.array_equal(o.round_to_bf16_bits(y), out["o"])
    gu = o.bf16_bits_to_f32(out["gate_up"]).astype(np.float64)
    h = gu[:, :ffn] * (1 / (1 + np.exp(-gu[:, :ffn]))) * gu[:, ffn:]
    assert np.array_equal(o.round_to_bf16_bits(h), out["h"])
    assert out["down"].shape == (m, hidden)
    # calibration: every scale is amax / 448 of that layer's bf16 input, so the input's largest element hits +-448
    cal = o.calibrate_block_scales(x, layers, g, hidden, ffn)
    out = o.block_ref(x, layers, cal, g, hidden, ffn)
    for nm in ("qkv", "o", "gate_up", "down"):
        assert (out[nm + "_x8"] & 0x7F).max() == 0x7E
    assert cal["qkv"] == o.act_scale_from_amax(o.bf16_bits_to_f32(x))
    # silu closed forms: silu(0) = 0, silu(x) -> x for large x, -> 0 for very negative x
    t = syn.f32_to_bf16_bits(np.array([[0.0, 40.0, -40.0, 1.0, 1.0, 1.0]], np.float32))
    r = o.silu_mul_ref(t, 3)[0]
    assert r[0] == 0 and r[1] == 40.0 and abs(r[2]) < 1e-15
