"""Pins for the oracle's offline calibration: the Hessian factor behind Eq. 12, DPQ (Alg. 1) and Group-Aware
Reordering (Sec. 3.2, App. A.3)."""
import numpy as np

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import synthetic as syn


def correlated_inputs(rng, t, k):
    """Calibration activations with unequal feature magnitudes and correlations between features."""
    base = rng.standard_normal((t, k))
    mix = np.eye(k) + 0.3 * rng.standard_normal((k, k)) / np.sqrt(k)
    return (base @ mix) * np.exp(rng.uniform(-1.0, 1.0, size=k))[None, :]


def layer_error(w, x, codes, scales, zeros, s_w, g):
    """|| (W - W_hat) X^T ||^2 with W_hat the weights inference will use (Eq. 10, 11)."""
    _, w8 = o.linear_ref_asym_paper_literal(np.zeros((1, w.shape[1]), np.uint8), 1.0, codes, zeros, scales,
                                            np.ones(w.shape[0]), g)
    w_hat = o.e4m3_decode(w8) * np.asarray(s_w, dtype=np.float64).reshape(-1, 1)
    return float(np.linalg.norm((w.astype(np.float64) - w_hat) @ x.T) ** 2)


def test_factor_rows_are_the_update_coefficients_of_eq12():
    """For every q: row q of the inverse Hessian of the remaining weights {q, ...}, divided by its diagonal entry,
    equals U[q, q:] / U[q, q] -- computed here by explicitly inverting each sub-Hessian."""
    rng = np.random.default_rng(71)
    x = correlated_inputs(rng, 64, 7)
    u = o.hessian_inverse_factor(x, damp=0.01)
    h = x.T @ x
    h = h + np.eye(7) * 0.01 * np.mean(np.diag(h))
    assert np.allclose(u.T @ u, np.linalg.inv(h), rtol=1e-9, atol=1e-12)
    assert np.allclose(u, np.triu(u))
    for q in range(7):
        sub = np.linalg.inv(h[q:, q:])
        assert np.allclose(sub[0] / sub[0, 0], u[q, q:] / u[q, q], rtol=1e-8, atol=1e-12)
        assert np.isclose(u[q, q] ** 2, sub[0, 0], rtol=1e-9)


def test_factor_from_a_formed_hessian_by_another_route():
    """H^-1 = U^T U with U upper triangular and a positive diagonal has one solution.  A route that never inverts H:
    the lower Cholesky factor L of the index-reversed dampened Hessian gives H = R R^T with R = (L reversed) upper
    triangular, and U = R^-1.  With a permutation the Hessian is that of the reordered columns."""
    rng = np.random.default_rng(74)
    k = 24
    x = correlated_inputs(rng, 200, k)
    h = x.T @ x
    perm = rng.permutation(k)
    for p in (None, perm):
        u = o.hessian_inverse_factor_from_h(h, damp=0.02, perm=p)
        hp = h if p is None else h[p][:, p]
        hd = hp + np.eye(k) * 0.02 * np.trace(hp) / k
        low = np.linalg.cholesky(hd[::-1, ::-1])
        r = low[::-1, ::-1]
        assert np.allclose(r, np.triu(r)) and np.allclose(r @ r.T, hd, rtol=1e-12)
        assert np.allclose(u, np.linalg.inv(r), rtol=1e-8, atol=1e-12)
        assert np.all(np.diag(u) > 0) and np.allclose(u, np.triu(u))
        assert np.allclose(u.T @ u @ hd, np.eye(k), atol=1e-8)
    assert np.array_equal(o.hessian_inverse_factor(x, 0.02), o.hessian_inverse_factor_from_h(h, 0.02))


def test_without_interactions_dpq_is_plain_double_quantization():
    """With U = I no error reaches another weight, and Alg. 1 reduces to its quantization steps alone: FP8 rounding
    (Eq. 7) followed by the asymmetric quantizer of Eq. 8-9 on the FP8 values -- the oracle's separately pinned
    asym_quantize_weights."""
    rng = np.random.default_rng(72)
    n, k, g = 24, 512, 128
    w = syn.make_weights(rng, n, k)
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    w8 = o.e4m3_decode(o.e4m3_encode((w / s_w[:, None]).astype(np.float32))).astype(np.float32)
    u0, s0, z0 = o.asym_quantize_weights(w8, g)
    codes, scales, zeros = o.dpq_quantize(w, np.eye(k, dtype=np.float32), s_w, g)
    assert np.array_equal(codes, u0) and np.array_equal(scales, s0) and np.array_equal(zeros, z0)
    # a column order does not matter either in that case, and the results come back in the original order
    perm = o.gar_permutation(rng.random(k), g)
    c2, s2, z2 = o.dpq_quantize(w, np.eye(k, dtype=np.float32), s_w, g, perm=perm)
    assert np.array_equal(c2, u0) and np.array_equal(s2, s0) and np.array_equal(z2, z0)


def test_updates_follow_eq12_with_explicit_sub_hessians():
    """A second statement of the algorithm on a tiny case, float64, that never forms the Cholesky factor: at each step
    the remaining weights move by -(w - w_hat) / [H_F^-1]_qq * (H_F^-1)_q,: with H_F the Hessian of the weights not yet
    quantized, inverted explicitly.  Codes and group parameters must agree with the float32 oracle; a row is followed
    until one of its rounding decisions comes next to a tie, where float32 and float64 weights may part ways."""
    rng = np.random.default_rng(73)
    n, k, g = 5, 8, 4
    x = correlated_inputs(rng, 40, k)
    h = x.T @ x
    h = h + np.eye(k) * 0.01 * np.mean(np.diag(h))
    w = (rng.standard_normal((n, k)) * 0.05).astype(np.float32)
    s_w = np.float32(2.0 ** -10)                                          # W / s_w lands mid-range of the FP8 grid
    codes, scales, zeros = o.dpq_quantize(w, o.hessian_inverse_factor(x), s_w, g)
    def nearest(v):
        """FP8 value of a float32 number (the E4M3 rounding is pinned on its own); also says whether the decision would
        survive a relative perturbation of 1e-5, i.e. is not next to a tie."""
        v = np.float32(v)
        r = [float(o.e4m3_decode(o.e4m3_encode(np.float32(v * f)))) for f in (1.0, 1.0 - 1e-5, 1.0 + 1e-5)]
        return r[0], r[0] == r[1] == r[2]

    checked = 0
    for row in range(n):
        cur = w[row].astype(np.float64).copy()
        robust = True
        for q in range(k):
            if q % g == 0:
                pairs = [nearest(v / float(s_w)) for v in cur[q:q + g]]
                w8g = np.array([p[0] for p in pairs])
                robust &= all(p[1] for p in pairs)
                lo, hi = min(w8g.min(), 0.0), max(w8g.max(), 0.0)
                s = float(np.float32(np.float32(hi - lo) / np.float32(15.0)))
                z = float(np.rint(np.float32(np.float32(-lo) / np.float32(s))))
                if robust:
                    assert s == scales[row, q // g] and z == zeros[row, q // g]
            w8, ok = nearest(cur[q] / float(s_w))
            lvl = float(np.float32(np.float32(np.float32(w8) / np.float32(s)) + np.float32(z)))
            robust &= ok and abs(lvl - np.floor(lvl) - 0.5) > 1e-3
            if not robust:
                break                                                  # a decision next to a tie: leave the row out
            u = min(max(np.rint(lvl), 0.0), 15.0)
            assert u == codes[row, q], (row, q)
            checked += 1
            w8_hat, _ = nearest(np.float32(np.float32(u - z) * np.float32(s)))        # an exact float32 tie is a tie for both
            sub = np.linalg.inv(h[q:, q:])
            cur[q:] = cur[q:] - (cur[q] - w8_hat * float(s_w)) / sub[0, 0] * sub[0]
    assert checked >= 3 * k


def test_compensation_lowers_the_layer_error_and_gar_keeps_groups():
    """The point of Alg. 1 (Eq. 5): on correlated calibration inputs the compensated weights reproduce the layer
    output better than the same double quantization without compensation; with GAR the scales still belong to the
    original groups (the inference format is unchanged) and the error does not grow on average."""
    g, n, k = 128, 32, 256
    plain, dpq, gar = [], [], []
    for seed in range(4):
        rng = np.random.default_rng([74, seed])
        x = correlated_inputs(rng, 512, k)
        w = syn.make_weights(rng, n, k)
        s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
        c0 = o.dpq_quantize(w, np.eye(k, dtype=np.float32), s_w, g)
        c1 = o.dpq_quantize(w, o.hessian_inverse_factor(x), s_w, g)
        perm = o.gar_permutation(np.diag(x.T @ x), g)
        c2 = o.dpq_quantize(w, o.hessian_inverse_factor(x[:, perm]), s_w, g, perm=perm)
        plain.append(layer_error(w, x, *c0, s_w, g))
        dpq.append(layer_error(w, x, *c1, s_w, g))
        gar.append(layer_error(w, x, *c2, s_w, g))
        assert dpq[-1] < 0.9 * plain[-1] and gar[-1] < 0.9 * plain[-1]
        for c in (c1, c2):
            assert c[0].max() <= 15 and c[2].max() <= 15 and np.all(c[1] > 0)
    assert np.mean(gar) <= 1.05 * np.mean(dpq)


def test_gar_permutation_hand_example_and_structure():
    # groups of three: maxima 5 and 9 -> the second group goes first; inside each group descending diagonal
    assert o.gar_permutation([1, 5, 3, 9, 2, 4], 3).tolist() == [3, 5, 4, 1, 2, 0]
    # ties keep the lower original index first
    assert o.gar_permutation([2, 2, 1, 1, 2, 2], 2).tolist() == [0, 1, 4, 5, 2, 3]
    rng = np.random.default_rng(75)
    d = rng.random(1024)
    p = o.gar_permutation(d, 128)
    assert sorted(p.tolist()) == list(range(1024))
    blocks = p.reshape(8, 128)
    assert np.all(blocks // 128 == (blocks[:, :1] // 128))                # every visited group is one original group
    assert np.all(np.diff(d[blocks], axis=1) <= 0)                        # descending inside a group
    assert np.all(np.diff(d[blocks[:, 0]]) <= 0)                          # groups by descending maximum
