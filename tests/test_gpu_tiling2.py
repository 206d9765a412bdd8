"""GPU parity of the second tiling of the many-token kernel (2-D grid of wavefronts, expansion shared through LDS,
persistent workgroups) and of its split of K across workgroups (Sec. 1: both regimes have to be served; Sec. 3, Eq. 10,
Eq. 4, Eq. 11: the layer itself), against the CPU oracle on the same seeded inputs: every workgroup tile, ragged edges,
persistent grids smaller than the tile count (several tiles per workgroup), group sizes of one or more chunks, the -8
marks, the exact-integer case bit for bit, power-of-two scales through the block-scaled MFMA, and w4a8_linear with a
workspace on the shapes w4a8_linear_workspace_bytes() names.  Tolerances as in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

from test_gpu_parity import bf16_bits, check_outputs, dev, host, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
POW2_PATH = 2 + 16 * 3
TILES = (0, 1, 2, 3, 4, 5)


def run_variant(x8_d, sx_d, packed, scales, n, g, path, p0, p1):
    m = x8_d.shape[0]
    y32 = torch.full((m, n), float("nan"), dtype=torch.float32, device=DEV)
    y16 = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.linear_variant(x8_d, sx_d, packed, scales, n, g, y32, path, p0, p1)
    B.linear_variant(x8_d, sx_d, packed, scales, n, g, y16, path, p0, p1)
    return host(y32), bf16_bits(y16)


def realistic(seed, m, k, n, g, frac=0.02):
    rng = np.random.default_rng(seed)
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, frac, 20.0)
    s_x = syn.static_act_scale(x)
    q, s_w = o.rtn_quantize_weights(w, g)
    x8 = o.quantize_act(x, s_x)
    ref, a = o.linear_ref(x8, s_x, q, s_w, g)
    packed, scales = B.pack_weights(dev(w), g, B.LAYOUT_TILED)
    return x8, s_x, packed, scales, ref, a


def integer_case(seed, m, k, n, g, minus_eight):
    """Small-integer activations and power-of-two scales: every partial sum is exact in float32 in any order, so the
    float32 output must equal the integer matmul bit for bit (also across a split of K)."""
    rng = np.random.default_rng(seed)
    ng = k // g
    xi = rng.integers(-4, 5, size=(m, k))
    x8 = o.e4m3_encode(xi.astype(np.float32))
    q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)
    if minus_eight:
        marked = rng.random((n, ng)) < 0.25
        marked[:16] = False
        for nn, gg in zip(*np.nonzero(marked)):
            q[nn, gg * g + rng.choice(g, size=rng.integers(1, 4), replace=False)] = -8
    e = rng.integers(-1, 2, size=(n, ng))
    s_w = np.ldexp(1.0, e).astype(np.float32)
    part = np.einsum("mgk,ngk->mng", xi.reshape(m, ng, g).astype(np.int64), q.reshape(n, ng, g).astype(np.int64))
    want = (0.5 * (part * np.ldexp(1.0, e)[None]).sum(axis=2)).astype(np.float32)
    packed, scales = B.pack_weights(dev(q), g, B.LAYOUT_TILED, dev(s_w))
    return x8, packed, scales, want


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("m,k,n,g,p1", [
    (300, 1024, 520, 512, 0), (513, 256, 144, 256, 0), (70, 128, 20, 128, 0), (257, 640, 130, 128, 0),
    # persistent grids of 8 and 16 workgroups: several tiles per workgroup, the next tile's start inside the epilogue
    (700, 384, 1100, 128, 1 | (8 << 8)), (1300, 640, 600, 128, 3 | (16 << 8)),
])
def test_every_tile_ragged_against_the_oracle(gpu_lib, tile, m, k, n, g, p1):
    x8, s_x, packed, scales, ref, a = realistic([71, m, k, n], m, k, n, g)
    y32, y16 = run_variant(dev(x8), dev(np.array([s_x])), packed, scales, n, g, 2, tile, p1)
    check_outputs(y32, y16, ref, a, f"second tiling, tile {tile}, {m}x{k}x{n} g{g} p1={p1}")


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("m,g,minus_eight,p1", [(200, 128, False, 0), (300, 256, True, 0), (600, 128, True, 2 | (8 << 8))])
def test_every_tile_exact_integer_case_bit_for_bit(gpu_lib, tile, m, g, minus_eight, p1):
    k, n = 2048, 304
    x8, packed, scales, want = integer_case([73, m, g], m, k, n, g, minus_eight)
    y32, _ = run_variant(dev(x8), dev(np.array([0.5], np.float32)), packed, scales, n, g, 2, tile, p1)
    assert np.array_equal(y32, want)


@pytest.mark.parametrize("tile", (1, 4, 5))
def test_power_of_two_scales_on_the_second_tiling(gpu_lib, tile):
    m, k, n, g = 520, 1024, 300, 128
    rng = np.random.default_rng([75, tile])
    w = syn.make_weights(rng, n, k) * np.exp(rng.uniform(-3.0, 3.0, size=(n, 1))).astype(np.float32)
    x = syn.make_activations(rng, m, k, 0.02, 20.0)
    s_x = syn.static_act_scale(x)
    x8 = o.quantize_act(x, s_x)
    q, s = o.rtn_quantize_weights_pow2(w, g)
    ref, a = o.linear_ref(x8, s_x, q, s, g)
    packed, scales = B.pack_weights(dev(w), g, B.LAYOUT_TILED, pow2=True)
    y32, y16 = run_variant(dev(x8), dev(np.array([s_x])), packed, scales, n, g, POW2_PATH, tile, 0)
    check_outputs(y32, y16, ref, a, f"power-of-two scales, tile {tile}")


def test_default_path_takes_the_second_tiling_on_large_grids(gpu_lib):
    """M = 2048 on a 4096-channel layer (activations as in the benchmark configs: 1 % of the channels x 20): w4a8_linear
    routes to the second tiling -- the same bits as the explicit variant, and as the first tiling (one weight band per
    wavefront), whose sums run in the same order."""
    m, k, n, g = 2048, 1024, 4096, 128
    x8, s_x, packed, scales, ref, a = realistic([77], m, k, n, g, frac=0.01)
    sx_d = dev(np.array([s_x]))
    y = B.linear(dev(x8), sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.float32)
    y32, y16 = run_variant(dev(x8), sx_d, packed, scales, n, g, 2, 4, 0)
    first, _ = run_variant(dev(x8), sx_d, packed, scales, n, g, 1, 16, 1)
    assert np.array_equal(host(y), y32) and np.array_equal(first, y32)
    check_outputs(y32, y16, ref, a, "default path, 2048 x 1024 x 4096")


# ------------------------------------------------------------------------------------------------ K ranges across workgroups
def run_splitk(x8_d, sx_d, packed, scales, n, g, tile, ksplit):
    m = x8_d.shape[0]
    ws = torch.empty(ksplit * m * ((n + 63) // 64 * 64) * 4, dtype=torch.uint8, device=DEV)
    y32 = torch.full((m, n), float("nan"), dtype=torch.float32, device=DEV)
    y16 = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.linear_splitk_variant(x8_d, sx_d, packed, scales, n, g, y32, tile, ksplit, ws)
    B.linear_splitk_variant(x8_d, sx_d, packed, scales, n, g, y16, tile, ksplit, ws)
    return host(y32), bf16_bits(y16)


@pytest.mark.parametrize("tile,ksplit", [(5, 2), (5, 3), (5, 8), (3, 2), (3, 5), (1, 4)])
@pytest.mark.parametrize("m,k,n,g", [(100, 2048, 200, 128), (65, 1152, 136, 128), (300, 1024, 520, 512)])
def test_split_k_ragged_against_the_oracle(gpu_lib, tile, ksplit, m, k, n, g):
    """K ranges that do not divide the chunk count evenly, groups spanning several chunks (a range may end inside a
    group: the group's scale then multiplies two partial sums), ragged tokens and channels."""
    x8, s_x, packed, scales, ref, a = realistic([79, m, k, n], m, k, n, g)
    y32, y16 = run_splitk(dev(x8), dev(np.array([s_x])), packed, scales, n, g, tile, ksplit)
    check_outputs(y32, y16, ref, a, f"split K, tile {tile}, {ksplit} ranges, {m}x{k}x{n} g{g}")


@pytest.mark.parametrize("tile,ksplit", [(5, 2), (5, 7), (3, 16), (1, 3)])
def test_split_k_exact_integer_case_bit_for_bit(gpu_lib, tile, ksplit):
    m, k, n, g = 130, 2048, 304, 128
    x8, packed, scales, want = integer_case([81, tile, ksplit], m, k, n, g, True)
    y32, _ = run_splitk(dev(x8), dev(np.array([0.5], np.float32)), packed, scales, n, g, tile, ksplit)
    assert np.array_equal(y32, want)


@pytest.mark.parametrize("m", [48, 96, 128, 400])
def test_linear_with_workspace_on_the_down_projection(gpu_lib, m):
    """The Llama-3-8B down projection (K = 14336, N = 4096) at batch sizes where w4a8_linear asks for a workspace (from 41
    tokens on; at 48 the layer without a workspace runs on the few-token kernel): sampled
    token rows x all channels against the oracle, bf16 == RNE(float32), and the same bits on a second call (the order
    of the ranges in the sum is fixed)."""
    k, n = syn.LLAMA3_8B["down"]
    g = 128
    need = B.linear_workspace_bytes(m, k, n, g)
    assert need > 0
    rng = np.random.default_rng([83, m])
    w = syn.make_weights(rng, n, k)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    s_x = syn.static_act_scale(x)
    q, s_w = o.rtn_quantize_weights(w, g)
    x8 = o.quantize_act(x, s_x)
    rows = np.unique(np.concatenate([[0, m - 1], rng.integers(0, m, size=14)]))
    ref, a = o.linear_ref(x8[rows], s_x, q, s_w, g)
    packed, scales = B.pack_weights(dev(w), g, B.LAYOUT_TILED)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    sx_d, x8_d = dev(np.array([s_x])), dev(x8)
    y32 = host(B.linear(x8_d, sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.float32, workspace=ws))
    y16 = bf16_bits(B.linear(x8_d, sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.bfloat16, workspace=ws))
    check_outputs(y32[rows], y16[rows], ref, a, f"down projection with workspace, M = {m}")
    again = host(B.linear(x8_d, sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.float32, workspace=ws))
    assert np.array_equal(again.view(np.uint32), y32.view(np.uint32))
    # without a workspace the layer takes the unsplit kernels: same tolerance, different order of the sum
    plain = host(B.linear(x8_d, sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.float32))
    ok, worst = o.within_tolerance(plain[rows], ref, a)
    say(f"  without workspace: worst err/bound = {worst:.3e}")
    assert ok


def test_linear_with_workspace_at_k_8192(gpu_lib):
    """K = 8192 takes K ranges across workgroups when that gives four or more of them: a narrow layer at 100 tokens through
    w4a8_linear with the workspace it asks for, every output against the oracle."""
    m, k, n, g = 100, 8192, 2048, 128
    need = B.linear_workspace_bytes(m, k, n, g)
    assert need > 0 and B.linear_launch_shape(m, k, n, g, True)[0] == 3 and B.linear_workspace_bytes(m, 4096, n, g) == 0
    x8, s_x, packed, scales, ref, a = realistic([85], m, k, n, g, frac=0.01)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    sx_d, x8_d = dev(np.array([s_x])), dev(x8)
    y32 = host(B.linear(x8_d, sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.float32, workspace=ws))
    y16 = bf16_bits(B.linear(x8_d, sx_d, packed, scales, n, g, B.LAYOUT_TILED, out_dtype=torch.bfloat16, workspace=ws))
    check_outputs(y32, y16, ref, a, "K = 8192 with workspace")
