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


def group_mse(w, codes, scales, zeros, s_w, g):
    """Per (row, group): sum (W8 - W8_hat)^2 with W8 = the FP8 values of W / s_w (Eq. 7) and W8_hat what inference
    computes from the stored codes (Eq. 10), through the separately pinned literal dequantization."""
    n, k = w.shape
    _, w8_hat = o.linear_ref_asym_paper_literal(np.zeros((1, k), np.uint8), 1.0, codes, zeros, scales, np.ones(n), g)
    w8 = o.e4m3_decode(o.e4m3_encode((w / np.asarray(s_w, np.float32).reshape(-1, 1)).astype(np.float32)))
    d = (w8 - o.e4m3_decode(w8_hat)) ** 2
    return d.reshape(n, k // g, g).sum(axis=2)


def test_mse_scale_search_never_raises_a_groups_own_error_and_helps_with_outliers():
    """Sec. 3.3's search, with U = I so that groups do not interact: the parameters it picks give every (row, group) an
    error no larger than Eq. 8's own range does (candidate 0 is that range), strictly smaller where a lone outlier
    stretches the range; without a grid it is Eq. 8."""
    rng = np.random.default_rng(75)
    n, k, g = 12, 256, 64
    w = syn.make_weights(rng, n, k)
    w[np.arange(n), rng.integers(0, k, n)] *= 6.0                          # one outlier per row
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    eye = np.eye(k, dtype=np.float32)
    plain = o.dpq_quantize(w, eye, s_w, g)
    for same in (o.dpq_quantize(w, eye, s_w, g, mse_grid=0), o.dpq_quantize(w, eye, s_w, g, mse_grid=1)):
        assert all(np.array_equal(a, b) for a, b in zip(plain, same))
    searched = o.dpq_quantize(w, eye, s_w, g, mse_grid=40, mse_max_shrink=0.8)
    e0, e1 = group_mse(w, *plain, s_w, g), group_mse(w, *searched, s_w, g)
    assert np.all(e1 <= e0 * (1 + 1e-6))
    assert np.mean(e1 < 0.9 * e0) > 0.2                                   # the groups that hold an outlier, at least
    assert np.all(searched[1] <= plain[1])                                # shrunk ranges only


def test_mse_scale_search_picks_the_best_candidate_by_brute_force():
    """Every candidate range of the grid, scored independently in float64 from the definition (shrink the range, Eq. 8,
    Eq. 9 with clipping, Eq. 10 on the FP8 grid): the oracle's choice has the smallest score, and is the first such."""
    rng = np.random.default_rng(76)
    n, k, g, grid, shrink = 12, 64, 32, 16, 0.6
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    w[:, 5] *= 4.0
    s_w = np.float32(2.0 ** -11)
    _, scales, zeros = o.dpq_quantize(w, np.eye(k, dtype=np.float32), s_w, g, mse_grid=grid, mse_max_shrink=shrink)
    w8 = o.e4m3_decode(o.e4m3_encode((w / s_w).astype(np.float32)))
    checked = 0
    for r in range(n):
        for gi in range(k // g):
            v = w8[r, gi * g:(gi + 1) * g]
            lo, hi = min(v.min(), 0.0), max(v.max(), 0.0)
            zr = -lo * 15.0 / (hi - lo)                                   # the zero-point before rounding, the same for every candidate
            if abs(zr - np.floor(zr) - 0.5) < 1e-3:
                continue                                                  # a tie that float32 and float64 may round apart
            scores, params = [], []
            for i in range(grid):
                p = 1.0 - i * shrink / grid
                s = (p * hi - p * lo) / 15.0
                z = float(np.clip(np.rint(-p * lo / s), 0, 15))
                u = np.clip(np.rint(v / s + z), 0, 15)
                back = o.e4m3_decode(o.e4m3_encode(((u - z) * s).astype(np.float32)))
                scores.append(float(np.sum((v - back) ** 2)))
                params.append((s, z))
            order = np.argsort(scores, kind="stable")
            if scores[order[1]] - scores[order[0]] < 1e-4 * max(scores[order[0]], 1e-12):
                continue                                                  # float32 and float64 scores may rank a near-tie apart
            s_best, z_best = params[order[0]]
            assert np.isclose(scales[r, gi], s_best, rtol=1e-6) and zeros[r, gi] == z_best
            checked += 1
    assert checked >= 8


def test_mse_scale_search_keeps_a_range_that_is_already_exact():
    """Weights whose FP8 values are the sixteen levels 0..15 of a unit grid: Eq. 8's own range reproduces them exactly
    (score 0), and the first candidate with the smallest score is that one -- s = 1, z = 0."""
    w = np.tile(np.arange(16, dtype=np.float32), (3, 8))                   # [3, 128], values exact in E4M3
    _, scales, zeros = o.dpq_quantize(w, np.eye(128, dtype=np.float32), np.float32(1.0), 128, mse_grid=25)
    assert np.all(scales == 1.0) and np.all(zeros == 0)
