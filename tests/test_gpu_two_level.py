"""GPU parity of the two-level mode (Eq. 6-11 read literally): FP8 weight bytes nearest_E4M3(code * s8) bit-exact
against the oracle, layer outputs within |y - ref| <= 2e-3 * max(|ref|, A / 16), and bit-for-bit on an exact-integer
special case; both kernels (few tokens, MFMA-tiled) through w4a8_linear_two_level.

The floor is wider than the code-exact mode's A / 64 because here BOTH operands span the whole E4M3 range: the FP8
matrix unit truncates the products of each group of eight about 14 bits below the largest of them, and with weights
up to 448 next to weights near 1 that costs up to 5.3e-5 * A on these inputs (1e-5 * A with integer-code weights);
the datapath's worst case is 7 * 2^-14 = 4.3e-4 * A.  2e-3 / 16 = 1.25e-4 * A lies between the two."""
import numpy as np
import pytest
import torch

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

FLOOR = 2.0 ** -4

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def two_level_inputs(w, g):
    """Offline side of Eq. 6-9 in its symmetric form, as test input: per-channel s_w = max|W| / 448, W8 = the E4M3
    values of W / s_w, per-group s8 = max|W8| / 7, codes = round(W8 / s8) in [-8, 7]."""
    n, k = w.shape
    s_w = (np.abs(w).max(axis=1) / np.float32(448.0)).astype(np.float32)
    s_w[s_w == 0] = 1.0
    w8 = o.e4m3_decode(o.e4m3_encode((w / s_w[:, None]).astype(np.float32))).astype(np.float32)
    grp = w8.reshape(n, k // g, g)
    s8 = (np.abs(grp).max(axis=2) / np.float32(7.0)).astype(np.float32)
    s8[s8 == 0] = 1.0
    q = np.clip(np.rint(grp / s8[:, :, None]), -8, 7).astype(np.int8).reshape(n, k)
    return q, s8, s_w


def run(x8, s_x, q, s8, s_w, g, per_tensor=False):
    n, k = q.shape
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s8))
    so = np.full(1, s_w[0], np.float32) if per_tensor else s_w
    y32 = B.linear_two_level(dev(x8), dev(np.array([s_x], np.float32)), packed, scales, dev(so), n, g, out_dtype=torch.float32)
    y16 = B.linear_two_level(dev(x8), dev(np.array([s_x], np.float32)), packed, scales, dev(so), n, g, out_dtype=torch.bfloat16)
    w8 = B.dequant_weights_two_level(packed, scales, n, k, g)
    return host(y32), host(y16.view(torch.int16)).view(np.uint16), host(w8)


def test_two_level_bytes_bit_exact_including_saturation_underflow_and_minus_eight(gpu_lib):
    rng = np.random.default_rng(31)
    n, k, g = 72, 1024, 128
    q = rng.integers(-8, 8, size=(n, k)).astype(np.int8)
    q[:16] = rng.integers(-7, 8, size=(16, k))                          # a band without -8 anywhere
    s8 = np.exp(rng.uniform(np.log(2.0 ** -12), np.log(80.0), size=(n, k // g))).astype(np.float32)
    s8[3, 2] = 0.0
    s8[5, 1] = 2.0 ** -10 / 3                                           # 3 * s8 sits on the tie between 0 and 2^-9
    s8[6, 0] = 64.0                                                     # 7 * 64 = 448 exactly; 8 * 64 saturates
    x8 = np.zeros((1, k), np.uint8)
    _, want = o.linear_ref_paper_literal(x8, np.float32(1), q, s8, np.ones(n, np.float32), g)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s8))
    got = host(B.dequant_weights_two_level(packed, scales, n, k, g))
    assert np.array_equal(got, want)
    assert (want & 0x7F).max() == 0x7E and ((want & 0x7F) == 0).any()   # saturation and zeros are both present


@pytest.mark.parametrize("m,k,n,g", [(1, 1024, 96, 128), (16, 2048, 200, 256), (40, 1024, 72, 128), (64, 512, 48, 512),
                                     (100, 384, 300, 128), (300, 1024, 520, 512), (257, 640, 130, 128), (600, 2048, 1024, 128)])
def test_two_level_linear_against_the_oracle(gpu_lib, m, k, n, g):
    rng = np.random.default_rng([33, m, k, n])
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q, s8, s_w = two_level_inputs(w, g)
    ref, want8 = o.linear_ref_paper_literal(x8, s_x, q, s8, s_w, g)
    a = float(np.float32(s_x)) * (np.abs(o.e4m3_decode(x8)) @ np.abs(o.e4m3_decode(want8)).T) * s_w.astype(np.float64)[None, :]
    y32, y16, w8 = run(x8, s_x, q, s8, s_w, g)
    assert np.array_equal(w8, want8)
    ok, worst = o.within_tolerance(y32, ref, a, floor=FLOOR)
    print(f"  two-level {m}x{k}x{n} g{g}: worst err/bound {worst:.3e}", flush=True)
    assert ok
    assert np.array_equal(y16, o.round_to_bf16_bits(y32.astype(np.float64)))
    # the quantization error of the scheme itself stays small against the unquantized layer (sanity of the inputs)
    full = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.linalg.norm(ref - full) / np.linalg.norm(full) < 0.25


@pytest.mark.parametrize("m", [3, 16, 48, 200, 700])
def test_two_level_exact_integer_case_bit_for_bit_and_per_tensor_scale(gpu_lib, m):
    """Power-of-two group scales keep code * s8 on the E4M3 grid, small-integer activations keep every partial sum an
    integer multiple of a power of two below 2^24: fp32 accumulation is exact and the output must equal the integer
    matmul bit for bit; -8 occurs in a quarter of the groups."""
    rng = np.random.default_rng([35, m])
    k, n, g = 2048, 176, 128
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)
    marked = rng.random((n, ng)) < 0.25
    for nn, gg in zip(*np.nonzero(marked)):
        q[nn, gg * g + rng.integers(0, g)] = -8
    e = rng.integers(-1, 3, size=(n, ng))
    s8 = np.ldexp(1.0, e).astype(np.float32)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), q.reshape(n, ng, g).astype(np.int64))
    acc = (part * np.ldexp(1.0, e)[None]).sum(axis=2)
    s_w = np.ldexp(1.0, rng.integers(-3, 2, size=n)).astype(np.float32)
    want = (0.5 * acc * s_w[None, :]).astype(np.float32)
    y32, _, _ = run(x8, np.float32(0.5), q, s8, s_w, g)
    assert np.array_equal(y32, want)
    s_t = np.full(n, 0.25, np.float32)
    y32t, _, _ = run(x8, np.float32(0.5), q, s8, s_t, g, per_tensor=True)
    assert np.array_equal(y32t, (0.5 * 0.25 * acc).astype(np.float32))


@pytest.mark.parametrize("m", [4, 1024])
def test_two_level_llama_qkv_shape_sampled(gpu_lib, m):
    k, n, g = 4096, 6144, 128
    rng = syn.rng_for(6, m, k, n)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q, s8, s_w = two_level_inputs(w, g)
    y32, _, _ = run(x8, s_x, q, s8, s_w, g)
    rows = np.sort(np.random.default_rng(m).choice(m, size=min(m, 24), replace=False))
    ref, w8 = o.linear_ref_paper_literal(x8[rows], s_x, q, s8, s_w, g)
    a = float(np.float32(s_x)) * (np.abs(o.e4m3_decode(x8[rows])) @ np.abs(o.e4m3_decode(w8)).T) * s_w.astype(np.float64)[None, :]
    ok, worst = o.within_tolerance(y32[rows], ref, a, floor=FLOOR)
    print(f"  two-level qkv M={m}: worst err/bound {worst:.3e}", flush=True)
    assert ok


# ---------------------------------------------------------------- the second tiling (2-D grid of wavefronts, persistent workgroups)
TILES = (0, 1, 2, 3, 4, 5)


def run_tile(x8, s_x, q, s8, s_w, g, tile, p1=0, per_tensor=False):
    n, k = q.shape
    m = x8.shape[0]
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s8))
    so = dev(np.full(1, s_w[0], np.float32) if per_tensor else s_w)
    sx = dev(np.array([s_x], np.float32))
    y32 = torch.full((m, n), float("nan"), dtype=torch.float32, device=DEV)
    y16 = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.linear_two_level_variant(dev(x8), sx, packed, scales, so, n, g, y32, tile, p1)
    B.linear_two_level_variant(dev(x8), sx, packed, scales, so, n, g, y16, tile, p1)
    return host(y32), host(y16.view(torch.int16)).view(np.uint16)


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("m,k,n,g,p1", [(300, 1024, 520, 512, 0), (513, 256, 144, 256, 0), (70, 128, 20, 128, 0),
                                        # persistent grids of 8 and 16 workgroups: several tiles per workgroup
                                        (700, 384, 1100, 128, 1 | (8 << 8)), (1300, 640, 600, 128, 3 | (16 << 8))])
def test_two_level_on_every_tile_of_the_second_tiling(gpu_lib, tile, m, k, n, g, p1):
    """Ragged tokens and channels, groups of one or more chunks, the expanding wavefront's scales (not the multiplying
    one's) and the per-channel output scale in the epilogue, against the oracle's literal reading."""
    rng = np.random.default_rng([37, m, k, n])
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q, s8, s_w = two_level_inputs(w, g)
    ref, want8 = o.linear_ref_paper_literal(x8, s_x, q, s8, s_w, g)
    a = float(np.float32(s_x)) * (np.abs(o.e4m3_decode(x8)) @ np.abs(o.e4m3_decode(want8)).T) * s_w.astype(np.float64)[None, :]
    y32, y16 = run_tile(x8, s_x, q, s8, s_w, g, tile, p1)
    ok, worst = o.within_tolerance(y32, ref, a, floor=FLOOR)
    print(f"  two-level, second tiling, tile {tile}, {m}x{k}x{n} g{g}: worst err/bound {worst:.3e}", flush=True)
    assert ok
    assert np.array_equal(y16, o.round_to_bf16_bits(y32.astype(np.float64)))


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("m,g,p1", [(200, 128, 0), (600, 256, 2 | (8 << 8))])
def test_two_level_exact_integer_case_on_every_tile_bit_for_bit(gpu_lib, tile, m, g, p1):
    """As above with -8 in a quarter of the groups (the marked groups take the slow expansion after the steps of a chunk,
    in the first chunk of a tile the one at its start), per-channel and per-tensor output scales; and the same bits as
    the first tiling gives through w4a8_linear_two_level."""
    rng = np.random.default_rng([39, m, g])
    k, n = 2048, 304
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)
    marked = rng.random((n, ng)) < 0.25
    marked[:16] = False
    marked[16:32, 0] = True                                             # the first chunk of a tile, too
    for nn, gg in zip(*np.nonzero(marked)):
        q[nn, gg * g + rng.choice(g, size=rng.integers(1, 4), replace=False)] = -8
    e = rng.integers(-1, 3, size=(n, ng))
    s8 = np.ldexp(1.0, e).astype(np.float32)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), q.reshape(n, ng, g).astype(np.int64))
    acc = (part * np.ldexp(1.0, e)[None]).sum(axis=2)
    s_w = np.ldexp(1.0, rng.integers(-3, 2, size=n)).astype(np.float32)
    y32, _ = run_tile(x8, np.float32(0.5), q, s8, s_w, g, tile, p1)
    assert np.array_equal(y32, (0.5 * acc * s_w[None, :]).astype(np.float32))
    y32t, _ = run_tile(x8, np.float32(0.5), q, s8, np.full(n, 0.25, np.float32), g, tile, p1, per_tensor=True)
    assert np.array_equal(y32t, (0.5 * 0.25 * acc).astype(np.float32))
    first, _, _ = run(x8, np.float32(0.5), q, s8, s_w, g)
    assert np.array_equal(first, y32)
