"""Parity of the other weight formats at the sizes bench.py times them: the gate|up layer of Llama-3-8B
(K = 4096, N = 28672) at 1 and at 8192 tokens, and one Llama-3-70B layer (the O projection, K = N = 8192) at 16 and
4096 tokens, for the two-level reading (Eq. 6-11), the asymmetric format (Eq. 8-9, Eq. 14), its two-level reading and
power-of-two scales (Sec. 2.2).  Codes, scales and zero-points are drawn directly (the layer's definition holds for any
of them; the quantizers have their own tests); 16 sampled token rows x 512 sampled channels (first and last band
included) against the oracle's layer of that format, in the launch configuration the library chooses by itself."""
import numpy as np
import pytest
import torch

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

from test_gpu_parity import dev, host

pytestmark = pytest.mark.gpu
G = 128
SHAPES = [(1, 4096, 28672), (8192, 4096, 28672), (16, 8192, 8192), (4096, 8192, 8192)]
TWO_LEVEL_FLOOR = 2.0 ** -4           # both operands span the whole E4M3 range (as in the two-level tests)


def sample(m, n, seed):
    pick = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, m - 1], pick.choice(m, size=min(m, 14), replace=False)]))
    cols = np.unique(np.concatenate([np.arange(16), np.arange(n - 16, n), pick.choice(n, size=480, replace=False)]))
    return rows, cols


def activations(seed, m, k):
    x = syn.make_activations(np.random.default_rng(seed), m, k, 0.01, 20.0)
    s_x = syn.static_act_scale(x)
    return o.quantize_act(x, s_x), s_x


def abs_terms(x8, s_x, w8, s_out):
    return float(np.float32(s_x)) * (np.abs(o.e4m3_decode(x8)) @ np.abs(o.e4m3_decode(w8)).T) * s_out.astype(np.float64)[None, :]


@pytest.mark.parametrize("m,k,n", SHAPES)
def test_two_level(gpu_lib, m, k, n):
    rng = np.random.default_rng([101, m, k, n])
    q = rng.integers(-7, 8, size=(n, k), dtype=np.int8)
    q[rng.integers(0, n, 2000), rng.integers(0, k, 2000)] = -8
    s8 = rng.uniform(2.0, 60.0, size=(n, k // G)).astype(np.float32)         # products up to 8 * 60: some saturate at 448
    s_w = rng.uniform(2e-4, 2e-3, size=n).astype(np.float32)
    x8, s_x = activations([102, m, k], m, k)
    packed, scales = B.pack_weights(dev(q), G, B.LAYOUT_TILED, dev(s8))
    y = host(B.linear_two_level(dev(x8), dev(np.array([s_x])), packed, scales, dev(s_w), n, G, out_dtype=torch.float32))
    rows, cols = sample(m, n, [103, m, n])
    ref, w8 = o.linear_ref_paper_literal(x8[rows], s_x, q[cols], s8[cols], s_w[cols], G)
    ok, worst = o.within_tolerance(y[np.ix_(rows, cols)], ref, abs_terms(x8[rows], s_x, w8, s_w[cols]), floor=TWO_LEVEL_FLOOR)
    print(f"  two-level M={m} K={k} N={n}: worst err/bound {worst:.3e}", flush=True)
    assert ok and np.isfinite(y).all()


@pytest.mark.parametrize("m,k,n", SHAPES)
def test_asymmetric_and_its_two_level_reading(gpu_lib, m, k, n):
    rng = np.random.default_rng([105, m, k, n])
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, k // G), dtype=np.uint8)
    s = rng.uniform(0.005, 0.02, size=(n, k // G)).astype(np.float32)
    x8, s_x = activations([106, m, k], m, k)
    sx_d, x8_d = dev(np.array([s_x])), dev(x8)
    rows, cols = sample(m, n, [107, m, n])
    packed, params = B.pack_weights_asym(dev(u), G, dev(s), dev(z))
    y = host(B.linear_asym(x8_d, sx_d, packed, params, n, G, out_dtype=torch.float32))
    ref, a = o.linear_ref_asym(x8[rows], s_x, u[cols], z[cols], s[cols], G)
    ok, worst = o.within_tolerance(y[np.ix_(rows, cols)], ref, a)
    print(f"  asymmetric M={m} K={k} N={n}: worst err/bound {worst:.3e}", flush=True)
    assert ok and np.isfinite(y).all()
    # the two-level reading: FP8-domain scales in the same records, one output scale per channel
    s8 = rng.uniform(1.0, 30.0, size=(n, k // G)).astype(np.float32)
    s_w = rng.uniform(2e-4, 2e-3, size=n).astype(np.float32)
    packed8, params8 = B.pack_weights_asym(dev(u), G, dev(s8), dev(z))
    y2 = host(B.linear_asym_two_level(x8_d, sx_d, packed8, params8, dev(s_w), n, G, out_dtype=torch.float32))
    ref2, w8 = o.linear_ref_asym_paper_literal(x8[rows], s_x, u[cols], z[cols], s8[cols], s_w[cols], G)
    ok, worst = o.within_tolerance(y2[np.ix_(rows, cols)], ref2, abs_terms(x8[rows], s_x, w8, s_w[cols]), floor=TWO_LEVEL_FLOOR)
    print(f"  asymmetric two-level M={m} K={k} N={n}: worst err/bound {worst:.3e}", flush=True)
    assert ok and np.isfinite(y2).all()


@pytest.mark.parametrize("m,k,n", SHAPES)
def test_power_of_two_scales(gpu_lib, m, k, n):
    rng = np.random.default_rng([109, m, k, n])
    q = rng.integers(-7, 8, size=(n, k), dtype=np.int8)
    q[rng.integers(0, n, 2000), rng.integers(0, k, 2000)] = -8
    s = np.ldexp(1.0, rng.integers(-9, -5, size=(n, k // G))).astype(np.float32)
    x8, s_x = activations([110, m, k], m, k)
    packed, scales = B.pack_weights(dev(q), G, B.LAYOUT_TILED, dev(s))
    y = host(B.linear_pow2(dev(x8), dev(np.array([s_x])), packed, scales, n, G, out_dtype=torch.float32))
    rows, cols = sample(m, n, [111, m, n])
    ref, a = o.linear_ref(x8[rows], s_x, q[cols], s[cols], G)
    ok, worst = o.within_tolerance(y[np.ix_(rows, cols)], ref, a)
    print(f"  power-of-two scales M={m} K={k} N={n}: worst err/bound {worst:.3e}", flush=True)
    assert ok and np.isfinite(y).all()
