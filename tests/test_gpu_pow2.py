"""GPU parity of the power-of-two-scale layer (Sec. 2.2: power-of-two scaling factors; here the group scale 2^e is
applied by the FP8 matrix unit itself, block-scaled MFMA): packed codes and scales bit-exact against the oracle's
power-of-two quantizer, layer outputs against the oracle's layer (the definition does not change: linear_ref with
power-of-two scales) within |y - ref| <= 2e-3 * max(|ref|, A / 64), bit for bit on an exact-integer case; both
kernels (few tokens, MFMA-tiled) through w4a8_linear_pow2."""
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


def sx_dev(s_x):
    return dev(np.array([s_x], np.float32))


@pytest.mark.parametrize("n,k,g,layout", [(200, 1024, 128, B.LAYOUT_TILED), (37, 512, 256, B.LAYOUT_TILED),
                                          (50, 256, 32, B.LAYOUT_CANONICAL)])
def test_pack_with_power_of_two_scales_bit_exact(gpu_lib, n, k, g, layout):
    rng = np.random.default_rng([51, n, k, g])
    w = syn.make_weights(rng, n, k)
    w[1, :g] = 0.0                                               # all-zero group: scale 1
    w[2, :g] = 0.0
    w[2, 5] = 0.875                                              # max|W| / 7 = 2^-3 exactly: the scale is 2^-3, not 2^-2
    q, s = o.rtn_quantize_weights_pow2(w, g)
    packed, scales = B.pack_weights(dev(w), g, layout, pow2=True)
    if layout == B.LAYOUT_TILED:
        assert np.array_equal(host(packed), o.pack_tiled(q))
        assert np.array_equal(host(scales).view(np.uint32), o.tile_scales(s, q).view(np.uint32))
    else:
        assert np.array_equal(host(packed).reshape(n, k // 2), o.pack_canonical(q))
        assert np.array_equal(host(scales).reshape(n, k // g), s)
    assert s[1, 0] == 1.0 and s[2, 0] == 0.125 and q[2, 5] == 7


@pytest.mark.parametrize("m,k,n,g", [(1, 1024, 96, 128), (4, 512, 40, 512), (16, 2048, 200, 256), (33, 1024, 72, 128),
                                     (40, 8192, 64, 128), (64, 512, 48, 128), (100, 384, 300, 128),
                                     (257, 640, 130, 128), (300, 1024, 520, 512), (600, 2048, 1024, 128)])
def test_linear_against_the_oracle(gpu_lib, m, k, n, g):
    rng = np.random.default_rng([53, m, k, n])
    w = syn.make_weights(rng, n, k)
    w *= np.exp(rng.uniform(-3.0, 3.0, size=(n, 1))).astype(np.float32)      # rows of different magnitude: exponents vary
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q, s = o.rtn_quantize_weights_pow2(w, g)
    ref, a = o.linear_ref(x8, s_x, q, s, g)
    packed, scales = B.pack_weights(dev(w), g, B.LAYOUT_TILED, pow2=True)
    y32 = host(B.linear_pow2(dev(x8), sx_dev(s_x), packed, scales, n, g, out_dtype=torch.float32))
    y16 = host(B.linear_pow2(dev(x8), sx_dev(s_x), packed, scales, n, g, out_dtype=torch.bfloat16).view(torch.int16))
    ok, worst = o.within_tolerance(y32, ref, a)
    print(f"  pow2 {m}x{k}x{n} g{g}: worst err/bound {worst:.3e}", flush=True)
    assert ok
    assert np.array_equal(y16.view(np.uint16), o.round_to_bf16_bits(y32.astype(np.float64)))
    assert len(np.unique(s)) >= 4                                # several different exponents were in play


@pytest.mark.parametrize("m", [3, 16, 48, 200, 700])
def test_exact_integer_case_bit_for_bit(gpu_lib, m):
    """Small-integer activations and codes, power-of-two scales: every partial sum is an integer multiple of a power
    of two below 2^24, so the accumulation inside the matrix unit is exact and the output equals the integer matmul
    bit for bit; -8 occurs in a quarter of the groups, exponents -6 .. 5."""
    rng = np.random.default_rng([55, m])
    k, n, g = 2048, 176, 128
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)
    marked = rng.random((n, ng)) < 0.25
    for nn, gg in zip(*np.nonzero(marked)):
        q[nn, gg * g + rng.integers(0, g)] = -8
    e = rng.integers(-6, 6, size=(n, 1)) + rng.integers(0, 3, size=(n, ng))  # within a row the exponents span 2
    s = np.ldexp(1.0, e).astype(np.float32)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), q.reshape(n, ng, g).astype(np.int64))
    want = (0.5 * (part * np.ldexp(1.0, e)[None]).sum(axis=2)).astype(np.float32)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s))
    y32 = host(B.linear_pow2(dev(x8), sx_dev(0.5), packed, scales, n, g, out_dtype=torch.float32))
    assert np.array_equal(y32, want)


@pytest.mark.parametrize("m", [8, 120])
def test_only_the_exponent_of_a_scale_is_read(gpu_lib, m):
    """Scales that are not powers of two act as the power of two below them (the documented behaviour)."""
    rng = np.random.default_rng([56, m])
    k, n, g = 1024, 64, 128
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)
    s = (rng.random((n, k // g), dtype=np.float32) + np.float32(0.25)) * np.float32(0.01)
    mant, expo = np.frexp(s)
    s_floor = np.ldexp(np.float32(1.0), expo - 1).astype(np.float32)
    ref, a = o.linear_ref(x8, s_x, q, s_floor, g)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s))
    y32 = host(B.linear_pow2(dev(x8), sx_dev(s_x), packed, scales, n, g, out_dtype=torch.float32))
    ok, worst = o.within_tolerance(y32, ref, a)
    assert ok, worst


@pytest.mark.parametrize("m,layer", [(4, "qkv"), (16, "down"), (1024, "qkv"), (2048, "down")])
def test_llama_shapes_sampled(gpu_lib, m, layer):
    k, n = syn.LLAMA3_8B[layer]
    g = 128
    rng = syn.rng_for(8, m, k, n)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    packed, scales = B.pack_weights(dev(w), g, B.LAYOUT_TILED, pow2=True)
    y32 = host(B.linear_pow2(dev(x8), sx_dev(s_x), packed, scales, n, g, out_dtype=torch.float32))
    pick = np.random.default_rng([m, n])
    rows = np.sort(pick.choice(m, size=min(m, 16), replace=False))
    cols = np.unique(np.concatenate([np.arange(16), np.arange(n - 16, n), pick.choice(n, size=480, replace=False)]))
    q, s = o.rtn_quantize_weights_pow2(w[cols], g)
    ref, a = o.linear_ref(x8[rows], s_x, q, s, g)
    ok, worst = o.within_tolerance(y32[np.ix_(rows, cols)], ref, a)
    print(f"  pow2 {layer} M={m}: worst err/bound {worst:.3e}", flush=True)
    assert ok
