"""GPU parity of the asymmetric format (unsigned 4-bit codes with per-group scale and zero-point; Eq. 1, Eq. 8-9,
Eq. 14): packed codes, parameter records and FP8 operand bytes bit-exact against the oracle; layer outputs within
|y - ref| <= 2e-3 * max(|ref|, A / 64) (the same bound as the signed-code layer: the operands are again exact
integers), bit for bit on an exact-integer case and against the signed-code layer where the two formats coincide;
both kernels (few tokens, MFMA-tiled) through w4a8_linear_asym."""
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


@pytest.mark.parametrize("n,k,g", [(200, 1024, 128), (37, 512, 256), (16, 384, 384), (130, 2048, 128)])
def test_pack_from_weights_bit_exact(gpu_lib, n, k, g):
    rng = np.random.default_rng([41, n, k, g])
    w = syn.make_weights(rng, n, k)
    w[1, :g] = 0.0                                               # an all-zero group
    w[2, :g] = np.abs(w[2, :g])                                  # a group with one sign only: zero-point 0
    w[3, k - g:] = -np.abs(w[3, k - g:])                         # zero-point 15
    u, s, z = o.asym_quantize_weights(w, g)
    packed, params = B.pack_weights_asym(dev(w), g)
    assert np.array_equal(host(packed), o.pack_tiled_asym(u))
    assert np.array_equal(host(params), o.tile_params_asym(s, z))
    assert z[2, 0] == 0 and z[3, -1] == 15 and s[1, 0] == 1.0


def test_pack_from_codes_and_operand_bytes_bit_exact(gpu_lib):
    rng = np.random.default_rng(42)
    n, k, g = 100, 1024, 128
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, k // g), dtype=np.uint8)
    s = rng.random((n, k // g), dtype=np.float32)
    packed, params = B.pack_weights_asym(dev(u), g, dev(s), dev(z))
    assert np.array_equal(host(packed), o.pack_tiled_asym(u))
    assert np.array_equal(host(params), o.tile_params_asym(s, z))
    got = host(B.dequant_weights_asym(packed, params, n, k, g))
    want = o.dequant_asym_to_e4m3(u, z, g)
    assert np.array_equal(got, want)
    pairs = set(zip(u.ravel().tolist(), np.repeat(z, g, axis=1).ravel().tolist()))
    assert len(pairs) == 256                                     # every (code, zero-point) pair occurred


def layer_case(seed, m, k, n, g, frac=0.02, mult=20.0):
    rng = np.random.default_rng(seed)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, frac, mult)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    u, s, z = o.asym_quantize_weights(w, g)
    return w, x, s_x, x8, u, s, z


@pytest.mark.parametrize("m,k,n,g", [(1, 1024, 96, 128), (4, 512, 40, 512), (16, 2048, 200, 256), (33, 1024, 72, 128),
                                     (40, 8192, 64, 128), (64, 512, 48, 128), (100, 384, 300, 128),
                                     (257, 640, 130, 128), (300, 1024, 520, 512), (600, 2048, 1024, 128)])
def test_linear_against_the_oracle(gpu_lib, m, k, n, g):
    w, x, s_x, x8, u, s, z = layer_case([43, m, k, n], m, k, n, g)
    ref, a = o.linear_ref_asym(x8, s_x, u, z, s, g)
    packed, params = B.pack_weights_asym(dev(w), g)
    y32 = host(B.linear_asym(dev(x8), sx_dev(s_x), packed, params, n, g, out_dtype=torch.float32))
    y16 = host(B.linear_asym(dev(x8), sx_dev(s_x), packed, params, n, g, out_dtype=torch.bfloat16).view(torch.int16))
    ok, worst = o.within_tolerance(y32, ref, a)
    print(f"  asym {m}x{k}x{n} g{g}: worst err/bound {worst:.3e}", flush=True)
    assert ok
    assert np.array_equal(y16.view(np.uint16), o.round_to_bf16_bits(y32.astype(np.float64)))
    # the format's own error against the unquantized layer stays small (sanity of the inputs)
    full = (o.e4m3_decode(x8) * float(s_x)) @ w.astype(np.float64).T
    assert np.linalg.norm(ref - full) / np.linalg.norm(full) < 0.15


@pytest.mark.parametrize("m", [3, 16, 48, 200, 700])
def test_exact_integer_case_bit_for_bit(gpu_lib, m):
    """Small-integer activations, power-of-two scales: every partial sum is an integer multiple of a power of two
    below 2^24, fp32 accumulation is exact and the output equals the integer matmul bit for bit; every zero-point
    0..15 occurs."""
    rng = np.random.default_rng([45, m])
    k, n, g = 2048, 176, 128
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, ng), dtype=np.uint8)
    e = rng.integers(-2, 2, size=(n, ng))
    s = np.ldexp(1.0, e).astype(np.float32)
    d = u.reshape(n, ng, g).astype(np.int64) - z[:, :, None].astype(np.int64)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), d)
    want = (0.5 * (part * np.ldexp(1.0, e)[None]).sum(axis=2)).astype(np.float32)
    packed, params = B.pack_weights_asym(dev(u), g, dev(s), dev(z))
    y32 = host(B.linear_asym(dev(x8), sx_dev(0.5), packed, params, n, g, out_dtype=torch.float32))
    assert len(np.unique(z)) == 16
    assert np.array_equal(y32, want)


@pytest.mark.parametrize("m", [300, 1000])
def test_coincides_with_the_signed_code_layer(gpu_lib, m):
    """Codes q + 8 with zero-point 8 are the signed codes q: in the MFMA-tiled kernel the same operand bytes reach the
    matrix unit and the same fp32 operations follow, so the two entry points agree to the last bit."""
    rng = np.random.default_rng([46, m])
    k, n, g = 1024, 208, 128
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    s = (rng.random((n, k // g), dtype=np.float32) + np.float32(0.5)) * np.float32(0.003)
    u = (q.astype(np.int16) + 8).astype(np.uint8)
    z = np.full((n, k // g), 8, np.uint8)
    p_sym, s_sym = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s))
    p_asym, par = B.pack_weights_asym(dev(u), g, dev(s), dev(z))
    y_sym = host(B.linear(dev(x8), sx_dev(s_x), p_sym, s_sym, n, g, B.LAYOUT_TILED, out_dtype=torch.float32))
    y_asym = host(B.linear_asym(dev(x8), sx_dev(s_x), p_asym, par, n, g, out_dtype=torch.float32))
    assert np.array_equal(y_sym, y_asym)


@pytest.mark.parametrize("m,layer", [(4, "qkv"), (16, "down"), (1024, "qkv")])
def test_llama_shapes_sampled(gpu_lib, m, layer):
    k, n = syn.LLAMA3_8B[layer]
    g = 128
    rng = syn.rng_for(7, m, k, n)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    packed, params = B.pack_weights_asym(dev(w), g)
    y32 = host(B.linear_asym(dev(x8), sx_dev(s_x), packed, params, n, g, out_dtype=torch.float32))
    pick = np.random.default_rng([m, n])
    rows = np.sort(pick.choice(m, size=min(m, 16), replace=False))
    cols = np.sort(np.concatenate([np.arange(16), np.arange(n - 16, n), pick.choice(n, size=480, replace=False)]))
    cols = np.unique(cols)
    u, s, z = o.asym_quantize_weights(w[cols], g)
    ref, a = o.linear_ref_asym(x8[rows], s_x, u, z, s, g)
    ok, worst = o.within_tolerance(y32[np.ix_(rows, cols)], ref, a)
    print(f"  asym {layer} M={m}: worst err/bound {worst:.3e}", flush=True)
    assert ok


# ---- the two-level reading of the asymmetric format (Eq. 8-11 literally) --------------------------------------------
TWO_LEVEL_FLOOR = 2.0 ** -4      # both operands span the whole E4M3 range; same allowance as the signed two-level layer


def literal_inputs(w, g):
    """Offline side of Eq. 6-9 as test input: per-channel s_w = max|W| / 448, W8 = the E4M3 values of W / s_w, per
    group (range extended to contain zero) s8 = (max W8 - min W8) / 15, z = round(-min W8 / s8),
    u = clamp(round(W8 / s8 + z), 0, 15): the oracle's asymmetric quantizer applied to W8."""
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    s_w[s_w == 0] = 1.0
    w8 = o.e4m3_decode(o.e4m3_encode((w / s_w[:, None]).astype(np.float32))).astype(np.float32)
    u, s8, z = o.asym_quantize_weights(w8, g)
    return u, z, s8, s_w


def test_two_level_bytes_bit_exact_with_saturation_ties_and_zero_scale(gpu_lib):
    rng = np.random.default_rng(47)
    n, k, g = 72, 1024, 128
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, k // g), dtype=np.uint8)
    s8 = np.exp(rng.uniform(np.log(2.0 ** -12), np.log(60.0), size=(n, k // g))).astype(np.float32)
    s8[3, 2] = 0.0
    s8[5, 1] = 2.0 ** -10 / 3                                           # 3 * s8 sits on the tie between 0 and 2^-9
    s8[6, 0] = 64.0                                                     # 7 * 64 = 448 exactly; 8 * 64 saturates
    z[6, 0] = 4
    _, want = o.linear_ref_asym_paper_literal(np.zeros((1, k), np.uint8), np.float32(1), u, z, s8, np.ones(n), g)
    packed, params = B.pack_weights_asym(dev(u), g, dev(s8), dev(z))
    got = host(B.dequant_weights_asym(packed, params, n, k, g, two_level=True))
    assert np.array_equal(got & 0x7F, want & 0x7F)
    nz = (want & 0x7F) != 0
    assert np.array_equal(got[nz], want[nz])                            # signs of all non-zero bytes
    assert (want & 0x7F).max() == 0x7E and (~nz).any()


@pytest.mark.parametrize("m,k,n,g", [(1, 1024, 96, 128), (16, 2048, 200, 256), (40, 1024, 72, 128), (64, 512, 48, 512),
                                     (100, 384, 300, 128), (300, 1024, 520, 512), (257, 640, 130, 128), (600, 2048, 1024, 128)])
def test_two_level_linear_against_the_oracle(gpu_lib, m, k, n, g):
    rng = np.random.default_rng([48, m, k, n])
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    u, z, s8, s_w = literal_inputs(w, g)
    ref, want8 = o.linear_ref_asym_paper_literal(x8, s_x, u, z, s8, s_w, g)
    a = float(np.float32(s_x)) * (np.abs(o.e4m3_decode(x8)) @ np.abs(o.e4m3_decode(want8)).T) * s_w.astype(np.float64)[None, :]
    packed, params = B.pack_weights_asym(dev(u), g, dev(s8), dev(z))
    y32 = host(B.linear_asym_two_level(dev(x8), sx_dev(s_x), packed, params, dev(s_w), n, g, out_dtype=torch.float32))
    y16 = host(B.linear_asym_two_level(dev(x8), sx_dev(s_x), packed, params, dev(s_w), n, g,
                                       out_dtype=torch.bfloat16).view(torch.int16))
    ok, worst = o.within_tolerance(y32, ref, a, floor=TWO_LEVEL_FLOOR)
    print(f"  asym two-level {m}x{k}x{n} g{g}: worst err/bound {worst:.3e}", flush=True)
    assert ok
    assert np.array_equal(y16.view(np.uint16), o.round_to_bf16_bits(y32.astype(np.float64)))
    full = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.linalg.norm(ref - full) / np.linalg.norm(full) < 0.25


@pytest.mark.parametrize("m", [3, 48, 200])
def test_two_level_exact_integer_case_bit_for_bit_and_per_tensor_scale(gpu_lib, m):
    rng = np.random.default_rng([49, m])
    k, n, g = 2048, 176, 128
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    u = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    z = rng.integers(0, 16, size=(n, ng), dtype=np.uint8)
    e = rng.integers(-1, 3, size=(n, ng))
    s8 = np.ldexp(1.0, e).astype(np.float32)
    d = u.reshape(n, ng, g).astype(np.int64) - z[:, :, None].astype(np.int64)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), d)
    acc = (part * np.ldexp(1.0, e)[None]).sum(axis=2)
    s_w = np.ldexp(1.0, rng.integers(-3, 2, size=n)).astype(np.float32)
    packed, params = B.pack_weights_asym(dev(u), g, dev(s8), dev(z))
    y32 = host(B.linear_asym_two_level(dev(x8), sx_dev(0.5), packed, params, dev(s_w), n, g, out_dtype=torch.float32))
    assert np.array_equal(y32, (0.5 * acc * s_w[None, :]).astype(np.float32))
    y32t = host(B.linear_asym_two_level(dev(x8), sx_dev(0.5), packed, params, dev(np.full(1, 0.25, np.float32)), n, g,
                                        out_dtype=torch.float32))
    assert np.array_equal(y32t, (0.5 * 0.25 * acc).astype(np.float32))
