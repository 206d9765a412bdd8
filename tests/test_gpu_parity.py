"""GPU parity: every step of the HIP path, called through the C-ABI, against the CPU oracle on the same seeded
inputs.  Integer and byte results (FP8 codes, INT4 codes, packed bytes, dequantized bytes) must be bit-exact;
layer outputs must satisfy |y - ref| <= 2e-3 * max(|ref|, A / 64) for fp32 outputs, where A is the sum of the
absolute terms; bf16 outputs must be the round-to-nearest-even of the fp32 output, and lie within half a bf16 ulp
(plus the same accumulation allowance scaled down) of the fp64 reference."""
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


def bf16_dev(bits):
    return dev(bits.view(np.int16)).view(torch.bfloat16)


def bf16_bits(t):
    return host(t.view(torch.int16)).view(np.uint16)


def say(msg):
    print(msg, flush=True)


def check_outputs(y_f32, y_bf16_bits, ref, a, label):
    ok, worst = o.within_tolerance(y_f32, ref, a)
    err = np.abs(y_f32 - ref)
    say(f"  {label}: fp32 worst err/bound = {worst:.3e}  max err/A = {np.max(err / np.maximum(a, 1e-300)):.2e}  "
        f"max|err|/max|ref| = {err.max() / np.abs(ref).max():.2e}")
    assert ok, label
    # bf16 kernel == RNE(bf16) of the fp32 kernel (same accumulation), checked with the oracle's rounding helper
    want_bits = o.round_to_bf16_bits(y_f32.astype(np.float64))
    assert np.array_equal(y_bf16_bits, want_bits), label + " bf16 != rne(fp32 result)"
    yb = o.bf16_bits_to_f32(y_bf16_bits).astype(np.float64)
    bound = o.bf16_half_ulp(np.maximum(np.abs(ref), np.abs(yb))) + 2e-3 * 2.0 ** -6 * a
    assert np.all(np.abs(yb - ref) <= bound), label + " bf16 vs reference"


# ------------------------------------------------------------------------------------------------ a1
def _act_cases():
    rng = np.random.default_rng(101)
    allbf = (np.arange(1 << 16, dtype=np.uint32) << 16).view(np.float32)
    grid = o.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mids = ((grid[:-1] + grid[1:]) / 2).astype(np.float32)
    near = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)),
                           grid.astype(np.float32)])
    near = np.concatenate([near, -near, np.array([448, 464, 465, 1e30, np.inf, -np.inf, 0.0, -0.0, 1e-30, -1e-30,
                                                  2.0 ** -10, 1e-45, -1e-45], dtype=np.float32)])
    rand = (rng.standard_normal(1 << 16) * np.exp(rng.uniform(-14, 8, 1 << 16))).astype(np.float32)
    return np.concatenate([allbf, near, rand])


def test_quantize_act_special_values_bit_exact(gpu_lib):
    x = _act_cases()
    pad = (-x.size) % 64
    x = np.concatenate([x, np.zeros(pad, np.float32)]).reshape(-1, 64)
    for s in (1.0, 0.37, 2.0 ** -7, 3.1e3):
        s32 = np.float32(s)
        want = o.quantize_act(x, s32)
        got = host(B.quantize_act(dev(x), dev(np.array([s32]))))
        nan = np.isnan(x)
        assert np.array_equal(got[~nan], want[~nan]), f"scale {s}"
        assert np.all((got[nan] & 0x7F) == 0x7F)                  # NaN in -> a NaN byte out (either sign)
    say("  quantize_act: all bf16 patterns, all midpoints +-1ulp, specials: bit-exact")


@pytest.mark.parametrize("m,k,ld,dtype", [(8, 1024, 1024, "f32"), (5, 1000, 1003, "f32"), (16, 4096, 4096, "bf16"),
                                          (3, 72, 80, "bf16"), (1, 14336, 14336, "f32"), (130, 4096, 4112, "bf16")])
def test_quantize_act_workload_bit_exact(gpu_lib, m, k, ld, dtype):
    rng = syn.rng_for(1, m, k)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    s = syn.static_act_scale(x)
    buf = np.zeros((m, ld), np.float32)
    buf[:, :k] = x
    if dtype == "bf16":
        bits = syn.f32_to_bf16_bits(buf)
        want = o.quantize_act(bits[:, :k], s, x_is_bf16_bits=True)
        xd = bf16_dev(bits)[:, :k]
    else:
        want = o.quantize_act(x, s)
        xd = dev(buf)[:, :k]
    out = torch.zeros((m, ld), dtype=torch.uint8, device=DEV)[:, :k]
    got = host(B.quantize_act(xd, dev(np.array([s])), out=out))
    assert np.array_equal(got, want)
    if dtype == "f32":
        assert (want & 0x7F).max() == 0x7E                        # the amax element sits on +-448


# ------------------------------------------------------------------------------------------------ a2, a3
@pytest.mark.parametrize("n,k,g", [(1024, 1024, 1024), (40, 384, 128), (16, 128, 128), (200, 2048, 256)])
def test_pack_rtn_bit_exact_both_layouts(gpu_lib, n, k, g):
    w = syn.make_weights(syn.rng_for(1, n, k), n, k)
    w[min(3, n - 1), :g] = 0.0                                    # an all-zero group
    q, s = o.rtn_quantize_weights(w, g)
    wd = dev(w)
    p_t, s_t = B.pack_weights(wd, g, B.LAYOUT_TILED)
    assert np.array_equal(host(p_t), o.pack_tiled(q))
    assert np.array_equal(host(s_t), o.tile_scales(s))
    p_c, s_c = B.pack_weights(wd, g, B.LAYOUT_CANONICAL)
    assert np.array_equal(host(p_c).reshape(n, k // 2), o.pack_canonical(q))
    assert np.array_equal(host(s_c).reshape(n, k // g), s)
    # Eq. 10 test hook: the bytes fed to the matrix unit
    want8 = o.dequant_codes_to_e4m3(q)
    assert np.array_equal(host(B.dequant_weights(p_t, n, k, B.LAYOUT_TILED)), want8)
    assert np.array_equal(host(B.dequant_weights(p_c, n, k, B.LAYOUT_CANONICAL)), want8)


def test_pack_codes_all_sixteen_values_and_small_groups(gpu_lib):
    rng = np.random.default_rng(5)
    n, k = 37, 256
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    q[0, :16] = np.arange(-8, 8)
    s = rng.uniform(0.001, 0.1, size=(n, k // 128)).astype(np.float32)
    p_t, s_t = B.pack_weights(dev(q), 128, B.LAYOUT_TILED, dev(s))
    assert np.array_equal(host(p_t), o.pack_tiled(q))
    want_s = o.tile_scales(s, q)                                  # sign bit marks the groups that hold -8
    assert np.signbit(want_s).any() and not np.signbit(want_s).all()
    assert np.array_equal(host(s_t).view(np.uint32), want_s.view(np.uint32))
    assert np.array_equal(host(B.dequant_weights(p_t, n, k, B.LAYOUT_TILED)), o.dequant_codes_to_e4m3(q))
    s32 = rng.uniform(0.001, 0.1, size=(n, k // 32)).astype(np.float32)
    p_c, s_c = B.pack_weights(dev(q), 32, B.LAYOUT_CANONICAL, dev(s32))
    assert np.array_equal(host(p_c).reshape(n, k // 2), o.pack_canonical(q))
    assert np.array_equal(host(s_c).reshape(n, k // 32), s32)
    assert np.array_equal(host(B.dequant_weights(p_c, n, k, B.LAYOUT_CANONICAL)), o.dequant_codes_to_e4m3(q))


# ------------------------------------------------------------------------------------------------ a4-a7
def run_linear(x8_d, sx_d, packed, scales, n, g, layout, variant=None):
    m = x8_d.shape[0]
    y32 = torch.full((m, n), float("nan"), dtype=torch.float32, device=DEV)
    y16 = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    if variant is None:
        B.linear(x8_d, sx_d, packed, scales, n, g, layout, out=y32)
        B.linear(x8_d, sx_d, packed, scales, n, g, layout, out=y16)
    else:
        B.linear_variant(x8_d, sx_d, packed, scales, n, g, y32, *variant)
        B.linear_variant(x8_d, sx_d, packed, scales, n, g, y16, *variant)
    return host(y32), bf16_bits(y16)


def test_config1_single_layer(gpu_lib):
    """M=8, K=N=1024, per-output-channel scales, fp32 output: both storage layouts."""
    (m, k, n) = syn.CONFIGS[1]["shapes"][0]
    w, x, s_x = syn.make_layer(1, 0, m, k, n)
    q, s_w = o.rtn_quantize_weights(w, k)
    x8 = o.quantize_act(x, s_x)
    ref, a = o.linear_ref(x8, s_x, q, s_w, k)
    sx_d = dev(np.array([s_x]))
    x8_d = B.quantize_act(dev(x), sx_d)
    assert np.array_equal(host(x8_d), x8)
    for layout in (B.LAYOUT_TILED, B.LAYOUT_CANONICAL):
        packed, scales = B.pack_weights(dev(w), k, layout)
        y32, y16 = run_linear(x8_d, sx_d, packed, scales, n, k, layout)
        check_outputs(y32, y16, ref, a, f"config 1 layout {layout}")


@pytest.mark.parametrize("m,k,n,g,path", [
    (1, 128, 16, 128, None), (5, 384, 40, 128, None), (16, 512, 200, 256, None), (37, 1024, 72, 128, None),
    (64, 256, 48, 256, None), (65, 384, 40, 128, None), (130, 512, 300, 128, None), (300, 1024, 520, 512, None),
    (7, 1024, 96, 128, (0, 1, 1)), (7, 1024, 96, 128, (0, 2, 3)), (20, 1024, 96, 128, (0, 4, 2)),
    (50, 2048, 144, 128, (0, 4, 4)), (33, 2048, 64, 128, (0, 1, 8)), (16, 2048, 64, 128, (0, 1, 16 + 2 * 256)),
    (3, 4096, 32, 128, (0, 1, 3 + 4 * 256)),
    # very wide layers from 17 tokens on: four bands per wavefront by default, the last workgroup short of bands
    (20, 256, 16400, 128, None), (32, 128, 16424, 128, None),
    # MFMA-tiled kernel: (path 1, 16-token blocks per workgroup, K-split groups); chunk counts that are not multiples
    # of the split (K = 384, 640, 1152), one-chunk K, group sizes spanning several chunks
    (9, 384, 40, 128, (1, 0, 0)), (9, 384, 40, 128, (1, 4, 1)), (129, 256, 272, 128, (1, 0, 0)),
    (100, 384, 300, 128, (1, 4, 2)), (100, 384, 300, 128, (1, 4, 4)), (70, 128, 20, 128, (1, 4, 4)),
    (300, 1024, 520, 512, (1, 8, 1)), (300, 1024, 520, 512, (1, 8, 2)), (300, 1152, 520, 128, (1, 8, 1)),
    (257, 384, 130, 128, (1, 16, 1)), (257, 640, 130, 128, (1, 8, 2)), (300, 1024, 520, 512, (1, 16, 1)),
    (70, 128, 20, 128, (1, 16, 1)), (513, 256, 144, 256, (1, 16, 1)), (513, 256, 144, 256, (1, 4, 1)),
    (200, 2560, 72, 256, (1, 8, 2)), (65, 640, 136, 128, (1, 4, 4)),
    (300, 1024, 520, 512, (1, 16, 1 + 2 * 256)), (257, 384, 130, 128, (1, 16, 1 + 2 * 256)), (70, 128, 20, 128, (1, 16, 1 + 2 * 256)),
])
def test_linear_small_ragged(gpu_lib, m, k, n, g, path):
    """Several tiles, ragged tails in M and N, group sizes of one or more chunks, both kernels."""
    rng = np.random.default_rng([7, m, k, n])
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    q, s_w = o.rtn_quantize_weights(w, g)
    x8 = o.quantize_act(x, s_x)
    ref, a = o.linear_ref(x8, s_x, q, s_w, g)
    sx_d = dev(np.array([s_x]))
    packed, scales = B.pack_weights(dev(w), g, B.LAYOUT_TILED)
    y32, y16 = run_linear(dev(x8), sx_d, packed, scales, n, g, B.LAYOUT_TILED, path)
    check_outputs(y32, y16, ref, a, f"ragged {m}x{k}x{n} g{g} {path}")


@pytest.mark.parametrize("m,path", [(3, None), (16, (0, 2, 4)), (48, None), (200, None), (200, (1, 4, 4)), (200, (1, 8, 2)), (200, (1, 16, 1)), (200, (1, 16, 1 + 2 * 256))])
def test_linear_exact_integer_case_bit_for_bit(gpu_lib, m, path):
    """Small-integer activations, all sixteen codes, power-of-two scales: every partial sum is an integer (or a
    dyadic rational) below 2^24, so fp32 accumulation is exact in any order and the fp32 output must equal the
    integer matmul bit for bit."""
    rng = np.random.default_rng([11, m])
    k, n, g = 2048, 176, 128
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    e = rng.integers(-1, 2, size=(n, k // g))
    s_w = np.ldexp(1.0, e).astype(np.float32)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, k // g, g).astype(np.int64), q.reshape(n, k // g, g).astype(np.int64))
    want = (0.5 * (part * np.ldexp(1.0, e)[None]).sum(axis=2)).astype(np.float32)
    ref, _ = o.linear_ref(x8, np.float32(0.5), q, s_w, g)
    assert np.array_equal(ref.astype(np.float32), want)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s_w))
    y32, _ = run_linear(dev(x8), dev(np.array([0.5], np.float32)), packed, scales, n, g, B.LAYOUT_TILED, path)
    assert np.array_equal(y32, want)


@pytest.mark.parametrize("m,g,path", [(1, 128, None), (16, 128, (0, 2, 4)), (40, 256, (0, 1, 8)), (64, 128, None), (200, 128, None),
                                      (200, 256, (1, 4, 4)), (200, 128, (1, 8, 2)), (300, 256, (1, 16, 1)), (300, 128, (1, 16, 1 + 2 * 256)),
                                      (100, 128, (1, 4, 2)), (130, 512, (1, 8, 1))])
def test_linear_minus_eight_in_some_groups_bit_for_bit(gpu_lib, m, g, path):
    """The tiled format stores -8 as the spare nibble 1000 and marks its (row, group) in the scale's sign bit; the
    kernels expand nibbles the short way except on marked chunks.  Codes in [-7, 7] with -8 sprinkled into a quarter
    of the (row, group) pairs (and into none of the first band), exact-integer inputs: marked and unmarked chunks
    meet in every wavefront, and the fp32 output must equal the integer matmul bit for bit."""
    rng = np.random.default_rng([17, m, g])
    k, n = 2048, 176
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)
    marked = rng.random((n, ng)) < 0.25
    marked[:16] = False
    for nn, gg in zip(*np.nonzero(marked)):
        pos = rng.choice(g, size=rng.integers(1, 4), replace=False)
        q[nn, gg * g + pos] = -8
    e = rng.integers(-1, 2, size=(n, ng))
    s_w = np.ldexp(1.0, e).astype(np.float32)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), q.reshape(n, ng, g).astype(np.int64))
    want = (0.5 * (part * np.ldexp(1.0, e)[None]).sum(axis=2)).astype(np.float32)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s_w))
    assert np.array_equal(host(packed), o.pack_tiled(q))
    assert np.array_equal(host(scales).view(np.uint32), o.tile_scales(s_w, q).view(np.uint32))
    assert np.array_equal(host(B.dequant_weights(packed, n, k, B.LAYOUT_TILED)), o.dequant_codes_to_e4m3(q))
    y32, _ = run_linear(dev(x8), dev(np.array([0.5], np.float32)), packed, scales, n, g, B.LAYOUT_TILED, path)
    assert np.array_equal(y32, want)


def test_linear_one_hot_positions(gpu_lib):
    """A single non-zero code per output channel, at a different k for every channel: the output is one activation
    times that code and scale -- any mismatch between the weight and activation operand order shows up here."""
    k, n, g, m = 512, 512, 128, 16
    rng = np.random.default_rng(13)
    q = np.zeros((n, k), np.int8)
    q[np.arange(n), np.arange(n)] = rng.integers(1, 8, size=n) * rng.choice([-1, 1], size=n)
    s_w = rng.uniform(0.5, 2.0, size=(n, k // g)).astype(np.float32)
    x8 = rng.integers(0, 0x7F, size=(m, k)).astype(np.uint8) | (rng.integers(0, 2, size=(m, k)).astype(np.uint8) << 7)
    ref, a = o.linear_ref(x8, np.float32(1.0), q, s_w, g)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s_w))
    y32, y16 = run_linear(dev(x8), dev(np.array([1.0], np.float32)), packed, scales, n, g, B.LAYOUT_TILED)
    want = (o.e4m3_decode(x8)[:, :n] * q[np.arange(n), np.arange(n)][None, :]).astype(np.float32) * \
        s_w[np.arange(n), np.arange(n) // g][None, :]
    assert np.array_equal(y32, want.astype(np.float32))
    check_outputs(y32, y16, ref, a, "one-hot")


# full-size layers: weights are quantized and packed once per (K, N) and shared by the decode and prefill cases
_LAYERS = {}


def full_layer(cfg_id, idx, k, n, n_rows=None):
    """Pack the full [N, K] layer on the GPU; run the oracle's quantizer on all rows, or on `n_rows` sampled output
    channels (always including the first and last 16) when the layer is too big for the host."""
    key = (cfg_id, k, n)
    if key not in _LAYERS:
        say(f"  building layer K={k} N={n}")
        w = syn.make_weights(syn.rng_for(cfg_id, idx, k, n), n, k)
        packed, scales = B.pack_weights(dev(w), 128, B.LAYOUT_TILED)
        if n_rows is None or n_rows >= n:
            rows = np.arange(n)
        else:
            r = np.random.default_rng([cfg_id, k, n]).choice(n - 32, size=n_rows - 32, replace=False) + 16
            rows = np.sort(np.concatenate([np.arange(16), r, np.arange(n - 16, n)]))
        q, s_w = o.rtn_quantize_weights(w[rows], 128)
        if rows.size == n:
            assert np.array_equal(host(packed), o.pack_tiled(q)), "packed bytes"
            assert np.array_equal(host(scales), o.tile_scales(s_w)), "scales"
        del w
        _LAYERS.clear()                                          # keep one layer resident at a time
        _LAYERS[key] = (packed, scales, rows, q, s_w)
    return _LAYERS[key]


def layer_case(cfg_id, idx, m, k, n, frac, mult, sample_m=None, n_rows=None):
    packed, scales, rows, q, s_w = full_layer(cfg_id, idx, k, n, n_rows)
    x = syn.make_activations(syn.rng_for(cfg_id, idx, m, k, n, 1), m, k, frac, mult)
    s_x = syn.static_act_scale(x)
    sx_d = dev(np.array([s_x]))
    x8_d = B.quantize_act(dev(x), sx_d)
    if sample_m is None or sample_m >= m:
        mrows = np.arange(m)
    else:
        r = np.random.default_rng([cfg_id, m]).choice(m - 2, size=sample_m - 2, replace=False) + 1
        mrows = np.sort(np.concatenate([[0], r, [m - 1]]))
    x8 = o.quantize_act(x[mrows], s_x)
    assert np.array_equal(host(x8_d)[mrows], x8), "x8"
    ref, a = o.linear_ref(x8, s_x, q, s_w, 128)
    y32, y16 = run_linear(x8_d, sx_d, packed, scales, n, 128, B.LAYOUT_TILED)
    check_outputs(y32[np.ix_(mrows, rows)], y16[np.ix_(mrows, rows)], ref, a, f"cfg{cfg_id} M={m} K={k} N={n}")
    assert np.isfinite(y32).all()


LLAMA8B = list(syn.LLAMA3_8B.values())
LLAMA70B = list(syn.LLAMA3_70B.values())


@pytest.mark.parametrize("idx", range(4))
def test_config2_config3_llama8b_full_shapes(gpu_lib, idx):
    """Decode (M = 1, 4, 16: every output checked), the sizes around the kernels' crossover and the K-split launch
    shapes (M = 33, 64, 128, 256) and prefill (M = 512, 2048, 8192) with 32 sampled token rows and all output
    channels, on the four Llama-3-8B layer shapes; one set of packed weights per shape."""
    k, n = LLAMA8B[idx]
    for m in (1, 4, 16):
        layer_case(2, idx, m, k, n, 0.01, 20.0)
    for m in (33, 64, 128, 256, 512, 2048, 8192):
        layer_case(2, idx, m, k, n, 0.01, 20.0, sample_m=32)


@pytest.mark.parametrize("idx", range(4))
def test_config4_llama70b_shapes_sampled(gpu_lib, idx):
    """Llama-3-70B shapes: 16 sampled token rows x 4096 sampled output channels (first and last tiles included)."""
    k, n = LLAMA70B[idx]
    for m in (1, 16, 4096):
        layer_case(4, idx, m, k, n, 0.005, 50.0, sample_m=16, n_rows=4096)


def test_silu_mul(gpu_lib):
    rng = np.random.default_rng(17)
    for m, f, ld in ((5, 1000, 2008), (32, 14336, 28672), (3, 7, 15)):
        gu = (rng.standard_normal((m, ld)) * 3).astype(np.float32)
        gu[0, :4] = [0.0, 80.0, -80.0, -0.0]
        bits = syn.f32_to_bf16_bits(gu)
        got = bf16_bits(B.silu_mul(bf16_dev(bits)[:, :2 * f]))
        ref = o.silu_mul_ref(bits[:, :2 * f], f)
        yb = o.bf16_bits_to_f32(got).astype(np.float64)
        # fp32 arithmetic then one bf16 rounding: half a bf16 ulp plus a few fp32 ulps
        assert np.all(np.abs(yb - ref) <= o.bf16_half_ulp(np.maximum(np.abs(ref), np.abs(yb))) * (1 + 2.0 ** -10) + 1e-30)
        assert np.mean(got == o.round_to_bf16_bits(ref)) > 0.995


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_act_scale_calibration_bit_exact(gpu_lib, dtype):
    """Eq. 13's scale over three calibration batches (one with a row stride, NaNs ignored) equals the oracle's
    act_scale_from_amax of all the values."""
    rng = np.random.default_rng(91)
    batches = [syn.make_activations(rng, m, 1000, 0.01, 20.0) for m in (1, 37, 300)]
    if dtype == "bf16":
        vals = [o.bf16_bits_to_f32(syn.f32_to_bf16_bits(b)) for b in batches]
        dev_batches = [torch.from_numpy(v).to(DEV).to(torch.bfloat16) for v in vals]
    else:
        vals = batches
        dev_batches = [torch.from_numpy(v).to(DEV) for v in vals]
    wide = torch.full((37, 1100), 1e9, dtype=dev_batches[1].dtype, device=DEV)
    wide[:, :1000] = dev_batches[1]
    dev_batches[1] = wide[:, :1000]                                       # strided rows; the padding must not be read
    nan_batch = dev_batches[0].clone()
    nan_batch[0, 5] = float("nan")
    got = B.calibrate_act_scale(dev_batches + [nan_batch])
    torch.cuda.synchronize()
    want = o.act_scale_from_amax(np.concatenate([v.ravel() for v in vals]))
    assert got.cpu().numpy()[0] == want


@pytest.mark.parametrize("m,k,n,dtype", [(1, 1024, 96, "f32"), (4, 512, 200, "bf16"), (16, 4096, 48, "f32"), (3, 14336, 40, "bf16"),
                                         (1, 4096, 6144, "bf16"), (4, 14336, 4096, "f32"), (9, 256, 520, "f32"),
                                         # launch shapes that differ from the common one: long rows on many bands (the plain
                                         # layer keeps four chunks in flight, this form two), grids between one and two
                                         # workgroups per compute unit (the plain layer takes four bands per wavefront,
                                         # this form two): the split of K has to stay the same
                                         (8, 8192, 8192, "bf16"), (2, 8192, 10240, "f32"), (16, 1024, 10240, "bf16")])
def test_linear_quantize_in_equals_the_two_calls(gpu_lib, m, k, n, dtype):
    """w4a8_linear_quantize_in: the FP8 codes it produces are the oracle's (Eq. 13), and its output is, bit for bit, that
    of w4a8_quantize_act followed by w4a8_linear; activations with a row stride, float32 and bf16, both output types."""
    rng = np.random.default_rng([31, m, k, n])
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    x[0, :4] = [1e9, -1e9, 0.0, -0.0]                                     # saturation and signed zero on the way
    s_x = syn.static_act_scale(x[:, 4:]) if k > 4 else np.float32(1.0)
    sx_d = dev(np.array([s_x], dtype=np.float32))
    packed, scales = B.pack_weights(dev(w), 128, B.LAYOUT_TILED)
    if dtype == "bf16":
        xb = syn.f32_to_bf16_bits(x)
        want8 = o.quantize_act(xb, s_x, x_is_bf16_bits=True)
        wide = torch.zeros((m, k + 64), dtype=torch.bfloat16, device=DEV)
        wide[:, :k] = torch.from_numpy(xb.view(np.int16)).to(DEV).view(torch.bfloat16)
    else:
        want8 = o.quantize_act(x, s_x)
        wide = torch.zeros((m, k + 64), dtype=torch.float32, device=DEV)
        wide[:, :k] = torch.from_numpy(x).to(DEV)
    x_d = wide[:, :k]
    x8 = B.quantize_act(x_d, sx_d)
    for out_dtype in (torch.float32, torch.bfloat16):
        two = B.linear(x8, sx_d, packed, scales, n, 128, B.LAYOUT_TILED, out_dtype=out_dtype)
        codes = torch.zeros((m, k), dtype=torch.uint8, device=DEV)
        one = B.linear_quantize_in(x_d, sx_d, packed, scales, n, 128, out_dtype=out_dtype, x8_out=codes)
        torch.cuda.synchronize()
        assert np.array_equal(codes.cpu().numpy(), want8)
        it = torch.int32 if out_dtype == torch.float32 else torch.int16
        assert torch.equal(one.view(it), two.view(it))
    assert np.array_equal(x8.cpu().numpy(), want8)
    # the form whose output is quantized for the next layer: the bytes of w4a8_quantize_act + w4a8_linear_fp8_out, which
    # in turn are the oracle's quantization (Eq. 13) of the bf16 output above
    y_scale = np.float32(max(float(two.abs().max()), 1e-3) / 448.0)
    ys_d = dev(np.array([y_scale], dtype=np.float32))
    two8 = B.linear_fp8_out(x8, sx_d, packed, scales, n, 128, ys_d)
    codes = torch.zeros((m, k), dtype=torch.uint8, device=DEV)
    wide8 = torch.zeros((m, n + 32), dtype=torch.uint8, device=DEV)
    one8 = B.linear_quantize_in_fp8_out(x_d, sx_d, packed, scales, n, 128, ys_d, out=wide8[:, :n], x8_out=codes)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), want8)
    assert torch.equal(one8, two8) and int(wide8[:, n:].max()) == 0
    assert np.array_equal(two8.cpu().numpy(), o.quantize_act(bf16_bits(two), y_scale, x_is_bf16_bits=True))
