"""GPU parity of the offline calibration: the Group-Aware Reordering permutation (Sec. 3.2, App. A.3) and Dual
Precision Quantization (Alg. 1) -- codes, group scales and zero-points bit-exact against the oracle, which takes the
same float32 steps -- and the calibrated weights through packing and the literal inference layer."""
import numpy as np
import pytest
import torch

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def calibration_inputs(rng, t, k):
    """Synthetic calibration activations: unequal feature magnitudes, mild correlations, a few outlier channels."""
    base = rng.standard_normal((t, k))
    mix = np.eye(k) + 0.3 * rng.standard_normal((k, k)) / np.sqrt(k)
    x = (base @ mix) * np.exp(rng.uniform(-1.0, 1.0, size=k))[None, :]
    x[:, rng.choice(k, size=max(1, k // 100), replace=False)] *= 20.0
    return x


@pytest.mark.parametrize("k,g", [(1024, 128), (512, 256), (384, 384)])
def test_gar_permutation_bit_exact(gpu_lib, k, g):
    rng = np.random.default_rng([81, k, g])
    d = rng.random(k).astype(np.float32)
    d[rng.choice(k, size=k // 8, replace=False)] = d[0]           # ties, inside groups and between group maxima
    if k > g:
        d[g:2 * g] = np.minimum(d[g:2 * g], d[:g].max())
        d[g + 3] = d[:g].max()
    got = host(B.gar_permutation(dev(d), g))
    assert np.array_equal(got, o.gar_permutation(d, g))


@pytest.mark.parametrize("n,k,g,per_channel,reorder", [(40, 256, 128, True, False), (150, 512, 256, True, True),
                                                       (70, 384, 128, False, True), (129, 640, 128, True, True)])
def test_dpq_bit_exact(gpu_lib, n, k, g, per_channel, reorder):
    rng = np.random.default_rng([82, n, k, g])
    w = syn.make_weights(rng, n, k)
    x = calibration_inputs(rng, 2 * k, k)
    perm = o.gar_permutation(np.diag(x.T @ x), g) if reorder else None
    u = o.hessian_inverse_factor(x[:, perm] if reorder else x).astype(np.float32)
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32) if per_channel else \
        np.array([np.abs(w).max() / np.float32(448.0)], dtype=np.float32)
    want = o.dpq_quantize(w, u, s_w, g, perm=perm)
    got = B.dpq_calibrate(dev(w), dev(u), dev(s_w), g, dev(perm.astype(np.int32)) if reorder else None)
    codes, scales, zeros = (host(t) for t in got)
    assert np.array_equal(scales, want[1]) and np.array_equal(zeros, want[2])
    assert np.array_equal(codes, want[0])
    # compensation took place: the codes differ from the uncompensated double quantization
    plain = o.dpq_quantize(w, np.eye(k, dtype=np.float32), s_w, g)
    assert np.mean(codes != plain[0]) > 0.05


@pytest.mark.parametrize("n,k,g,grid,shrink,reorder", [(40, 256, 128, 20, 0.8, False), (70, 512, 256, 37, 0.5, True),
                                                        (33, 384, 128, 5, 0.9, True), (17, 256, 128, 2, 0.3, False)])
def test_dpq_with_the_mse_scale_search_bit_exact(gpu_lib, n, k, g, grid, shrink, reorder):
    """Alg. 1 with the scale search of Sec. 3.3: candidates split over the lanes of a row on the GPU, scanned one after
    the other in the oracle -- the same float32 scores, the same first minimum, the same codes and parameters."""
    rng = np.random.default_rng([87, n, k, g])
    w = syn.make_weights(rng, n, k)
    w[np.arange(n), rng.integers(0, k, n)] *= 5.0                          # a stretched range in one group per row
    x = calibration_inputs(rng, 2 * k, k)
    perm = o.gar_permutation(np.diag(x.T @ x), g) if reorder else None
    u = o.hessian_inverse_factor(x[:, perm] if reorder else x).astype(np.float32)
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    want = o.dpq_quantize(w, u, s_w, g, perm=perm, mse_grid=grid, mse_max_shrink=shrink)
    got = B.dpq_calibrate(dev(w), dev(u), dev(s_w), g, dev(perm.astype(np.int32)) if reorder else None, mse_grid=grid,
                          mse_max_shrink=shrink)
    codes, scales, zeros = (host(t) for t in got)
    assert np.array_equal(scales, want[1]) and np.array_equal(zeros, want[2])
    assert np.array_equal(codes, want[0])
    plain = o.dpq_quantize(w, u, s_w, g, perm=perm)
    assert np.mean(scales != plain[1]) > 0.1                               # the search did move scales


def test_calibrated_weights_through_packing_and_inference(gpu_lib):
    """Calibration -> w4a8_pack_weights_asym -> w4a8_linear_asym_two_level: the layer on calibrated weights is closer
    to the unquantized layer, on the calibration inputs, than the layer on uncompensated weights; and the inference
    output matches the oracle's literal layer on the same codes."""
    rng = np.random.default_rng(83)
    n, k, g, t = 96, 512, 128, 1024
    w = syn.make_weights(rng, n, k)
    x = calibration_inputs(rng, t, k)
    s_x = syn.static_act_scale(x.astype(np.float32))
    x8 = o.quantize_act(x.astype(np.float32), s_x)
    xq = o.e4m3_decode(x8) * float(s_x)                                   # the activations inference sees
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    h_diag = np.diag(xq.T @ xq).astype(np.float32)
    perm = host(B.gar_permutation(dev(h_diag), g))
    u = o.hessian_inverse_factor(xq[:, perm]).astype(np.float32)
    full = xq @ w.astype(np.float64).T
    errs = {}
    for name, (uf, pm) in {"plain": (np.eye(k, dtype=np.float32), None), "dpq_gar": (u, perm)}.items():
        codes, scales, zeros = B.dpq_calibrate(dev(w), dev(uf), dev(s_w), g, dev(pm) if pm is not None else None)
        packed, params = B.pack_weights_asym(codes, g, scales, zeros)
        y = host(B.linear_asym_two_level(dev(x8), dev(np.array([s_x], np.float32)), packed, params, dev(s_w), n, g,
                                         out_dtype=torch.float32))
        ref, w8 = o.linear_ref_asym_paper_literal(x8, s_x, host(codes), host(zeros), host(scales), s_w, g)
        a = float(s_x) * (np.abs(o.e4m3_decode(x8)) @ np.abs(o.e4m3_decode(w8)).T) * s_w.astype(np.float64)[None, :]
        ok, worst = o.within_tolerance(y, ref, a, floor=2.0 ** -4)
        assert ok, (name, worst)
        errs[name] = float(np.linalg.norm(y - full) ** 2)
    print(f"  layer error on the calibration inputs: uncompensated {errs['plain']:.4e}, DPQ + GAR {errs['dpq_gar']:.4e}", flush=True)
    assert errs["dpq_gar"] < 0.9 * errs["plain"]


@pytest.mark.parametrize("t,k,dtype", [(1, 64, "f32"), (100, 200, "f32"), (1000, 384, "bf16"), (4096, 1024, "f32")])
def test_hessian_accumulate(gpu_lib, t, k, dtype):
    """H = X^T X over two batches (float32 accumulation on the GPU) against the float64 product of the same values:
    each entry within 2e-5 of sqrt(H_ii H_jj) (about a hundred float32 roundings of terms no larger than that)."""
    rng = np.random.default_rng([84, t, k])
    x = calibration_inputs(rng, 2 * t, k).astype(np.float32)
    if dtype == "bf16":
        x = o.bf16_bits_to_f32(syn.f32_to_bf16_bits(x))
        xd = torch.from_numpy(x).to(DEV).to(torch.bfloat16)
    else:
        xd = torch.from_numpy(x).to(DEV)
    wide = torch.full((t, k + 7), 1e6, dtype=xd.dtype, device=DEV)
    wide[:, :k] = xd[t:]
    h = B.hessian_accumulate(xd[:t])
    h = B.hessian_accumulate(wide[:, :k], h)                              # second batch with a row stride
    got = host(h).astype(np.float64)
    want = x.astype(np.float64).T @ x.astype(np.float64)
    d = np.sqrt(np.diag(want))
    assert np.all(np.abs(got - want) <= 2e-5 * np.outer(d, d) + 1e-30)
    assert np.array_equal(got, got.T)                                     # the same products in the same order


@pytest.mark.parametrize("k,reorder,damp", [(128, False, 0.01), (512, True, 0.01), (1024, True, 0.05), (1152, False, 0.01)])
def test_hessian_inverse_factor(gpu_lib, k, reorder, damp):
    """Dampening + Cholesky (Sec. 3.3) on the GPU (float64 inside) against the oracle's float64 route through the
    explicit inverse, from the same float32 Hessian: float32 rounding of the result plus a conditioning allowance."""
    rng = np.random.default_rng([85, k])
    x = calibration_inputs(rng, 2 * k, k)
    h = (x.T @ x).astype(np.float32)
    h = np.maximum(h, h.T)                                                # symmetric after the rounding to float32
    perm = o.gar_permutation(np.diag(h), 128) if reorder else None
    want = o.hessian_inverse_factor_from_h(h, damp, perm)
    u, info = B.hessian_inverse_factor(dev(h), damp, dev(perm.astype(np.int32)) if reorder else None)
    got = host(u).astype(np.float64)
    assert int(host(info)[0]) == 0
    assert np.all(np.tril(got, -1) == 0.0) and np.all(np.diag(got) > 0)
    assert np.all(np.abs(got - want) <= 2.0 ** -23 * np.abs(want) + 1e-9 * np.abs(want).max())
    hd = (h if perm is None else h[perm][:, perm]).astype(np.float64)
    hd = hd + np.eye(k) * damp * np.trace(hd) / k
    assert np.abs(got.T @ got @ hd - np.eye(k)).max() < 1e-3            # float32 entries of U: ~cond * 2^-24


def test_hessian_inverse_factor_reports_a_matrix_that_is_not_positive_definite(gpu_lib):
    k = 256
    h = np.eye(k, dtype=np.float32)
    h[100, 100] = -1.0
    _, info = B.hessian_inverse_factor(dev(h), 0.0)
    assert int(host(info)[0]) == k - 100                                  # 1 + index counted from the end: 155 + 1


def test_calibration_pipeline_on_the_gpu(gpu_lib):
    """Activations -> Hessian -> reordering -> factor -> Alg. 1, every step on the GPU, against the oracle run on the
    GPU's float32 Hessian: the permutation is identical; the factor agrees to float32 rounding, so all but a few codes
    (a decision next to a tie can flip, and its compensation moves a few later ones) are identical and the layer error
    is the same."""
    rng = np.random.default_rng(86)
    n, k, g, t = 64, 512, 128, 2048
    w = syn.make_weights(rng, n, k)
    x = calibration_inputs(rng, t, k).astype(np.float32)
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    h_d = B.hessian_accumulate(dev(x))
    perm_d = B.gar_permutation(torch.diagonal(h_d).contiguous(), g)
    u_d, info = B.hessian_inverse_factor(h_d, 0.01, perm_d)
    codes, scales, zeros = (host(a) for a in B.dpq_calibrate(dev(w), u_d, dev(s_w), g, perm_d))
    assert int(host(info)[0]) == 0
    h = host(h_d)
    perm = o.gar_permutation(np.diag(h), g)
    assert np.array_equal(host(perm_d), perm)
    u = o.hessian_inverse_factor_from_h(h, 0.01, perm).astype(np.float32)
    want = o.dpq_quantize(w, u, s_w, g, perm=perm)
    same = float(np.mean(codes == want[0]))
    print(f"  codes identical to the oracle's: {same:.5f}", flush=True)
    assert same > 0.995 and np.mean(zeros == want[2]) > 0.99

    def layer_error(c, s, z):
        _, w8 = o.linear_ref_asym_paper_literal(np.zeros((1, k), np.uint8), 1.0, c, z, s, np.ones(n), g)
        return float(np.linalg.norm((w.astype(np.float64) - o.e4m3_decode(w8) * s_w.astype(np.float64)[:, None]) @ x.T.astype(np.float64)) ** 2)
    e_gpu, e_ref = layer_error(codes, scales, zeros), layer_error(*want)
    plain = o.dpq_quantize(w, np.eye(k, dtype=np.float32), s_w, g)
    e_plain = layer_error(*plain)
    print(f"  layer error: GPU pipeline {e_gpu:.4e}, oracle {e_ref:.4e}, uncompensated {e_plain:.4e}", flush=True)
    assert abs(e_gpu - e_ref) < 0.02 * e_ref and e_gpu < 0.9 * e_plain


def test_calibration_at_the_size_bench_times_sampled_rows(gpu_lib):
    """A 4096 x 4096 layer with 8192 calibration tokens, the shapes of bench.py's calibration leg.  The factor from the
    GPU against the oracle's at full size; then Alg. 1 with GAR and the scale search on all 4096 rows on the GPU against
    the oracle on 12 sampled rows (rows are independent), bit for bit, both on the oracle's factor."""
    rng = np.random.default_rng(88)
    n = k = 4096
    g, t = 128, 8192
    print("  inputs", flush=True)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, t, k, 0.01, 20.0) * np.exp(rng.uniform(-1.0, 1.0, size=k)).astype(np.float32)[None, :]
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    h_d = B.hessian_accumulate(dev(x.astype(np.float32)))
    perm_d = B.gar_permutation(torch.diagonal(h_d).contiguous(), g)
    u_d, info = B.hessian_inverse_factor(h_d, 0.01, perm_d)
    h, perm = host(h_d), host(perm_d)
    assert int(host(info)[0]) == 0 and np.array_equal(perm, o.gar_permutation(np.diag(h), g))
    print("  oracle factor", flush=True)
    u = o.hessian_inverse_factor_from_h(h, 0.01, perm)
    got_u = host(u_d).astype(np.float64)
    assert np.all(np.abs(got_u - u) <= 2.0 ** -23 * np.abs(u) + 1e-9 * np.abs(u).max())
    u32 = u.astype(np.float32)
    print("  Alg. 1 on the GPU", flush=True)
    codes, scales, zeros = (host(a) for a in B.dpq_calibrate(dev(w), dev(u32), dev(s_w), g, perm_d, mse_grid=8, mse_max_shrink=0.6))
    rows = np.sort(np.concatenate([[0, n - 1], rng.choice(n - 2, 10, replace=False) + 1]))
    print("  Alg. 1 in the oracle, 12 rows", flush=True)
    want = o.dpq_quantize(w[rows], u32, s_w[rows], g, perm=perm, mse_grid=8, mse_max_shrink=0.6)
    assert np.array_equal(scales[rows], want[1]) and np.array_equal(zeros[rows], want[2])
    assert np.array_equal(codes[rows], want[0])


def test_hessian_inverse_factor_special_cases(gpu_lib):
    """A diagonal Hessian without dampening has the closed form U = diag(1 / sqrt(h_ii)); the identity permutation is
    the same as none; a reversal of the columns gives the factor of the reversed matrix."""
    rng = np.random.default_rng(89)
    k = 256
    d = rng.uniform(0.5, 4.0, k).astype(np.float32)
    u, info = B.hessian_inverse_factor(dev(np.diag(d)), 0.0)
    assert int(host(info)[0]) == 0
    assert np.allclose(host(u), np.diag(1.0 / np.sqrt(d.astype(np.float64))), rtol=2e-7, atol=0)
    x = calibration_inputs(rng, 2 * k, k)
    h = (x.T @ x).astype(np.float32)
    h = np.maximum(h, h.T)
    u0 = host(B.hessian_inverse_factor(dev(h), 0.01)[0])
    u1 = host(B.hessian_inverse_factor(dev(h), 0.01, dev(np.arange(k, dtype=np.int32)))[0])
    assert np.array_equal(u0, u1)
    rev = np.arange(k - 1, -1, -1, dtype=np.int32)
    u2 = host(B.hessian_inverse_factor(dev(h), 0.01, dev(rev))[0])
    u3 = host(B.hessian_inverse_factor(dev(np.ascontiguousarray(h[::-1, ::-1])), 0.01)[0])
    assert np.array_equal(u2, u3)


@pytest.mark.parametrize("n", [9000, 17000])
def test_dpq_many_rows_sampled(gpu_lib, n):
    """Layers with more than 8192 / 16384 rows run the block kernel with 16 / 8 lanes per row (and, beyond 16384, with U
    read from global memory): the same bits as the oracle on sampled rows, scale search included."""
    rng = np.random.default_rng([90, n])
    k, g = 256, 128
    w = syn.make_weights(rng, n, k)
    x = calibration_inputs(rng, 2 * k, k)
    perm = o.gar_permutation(np.diag(x.T @ x), g)
    u = o.hessian_inverse_factor(x[:, perm]).astype(np.float32)
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    got = B.dpq_calibrate(dev(w), dev(u), dev(s_w), g, dev(perm.astype(np.int32)), mse_grid=6, mse_max_shrink=0.5)
    codes, scales, zeros = (host(t) for t in got)
    rows = np.sort(np.concatenate([[0, n - 1], rng.choice(n - 2, 30, replace=False) + 1]))
    want = o.dpq_quantize(w[rows], u, s_w[rows], g, perm=perm, mse_grid=6, mse_max_shrink=0.5)
    assert np.array_equal(scales[rows], want[1]) and np.array_equal(zeros[rows], want[2])
    assert np.array_equal(codes[rows], want[0])
