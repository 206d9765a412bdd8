"""Run-to-run stability: every linear path launched 20 times in one process on fixed inputs must give identical bytes
(no path uses floating-point atomics; sums across wavefronts, K-split groups and K ranges are taken in a fixed order).
Stops at the first difference.  Covers the hazards a double-buffered kernel can have between its stages: a race would
show as an occasional different byte."""
import numpy as np
import pytest
import torch

from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
G = 128
REPEATS = 20


def inputs(seed, m, k, n):
    rng = np.random.default_rng(seed)
    w = torch.from_numpy(syn.make_weights(rng, n, k)).to(DEV)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    sx = torch.tensor([syn.static_act_scale(x)], dtype=torch.float32, device=DEV)
    xd = torch.from_numpy(x).to(DEV)
    return w, xd, B.quantize_act(xd, sx), sx


def repeat_and_compare(label, run):
    first = run().clone()
    torch.cuda.synchronize()
    for r in range(1, REPEATS):
        again = run()
        torch.cuda.synchronize()
        same = torch.equal(again.view(torch.uint8), first.view(torch.uint8))
        assert same, f"{label}: launch {r} differs from launch 0"
    print(f"  {label}: {REPEATS} launches, identical bytes", flush=True)


PATHS = [
    # label, M, K, N, (path, param0, param1) of w4a8_linear_variant or None for the default dispatch
    ("skinny, 1 token", 1, 4096, 1024, None), ("skinny, 16 tokens, 16 wavefronts", 16, 4096, 512, (0, 1, 16)),
    ("skinny, 48 tokens", 48, 2048, 768, None),
    ("first tiling 16/1/1", 600, 1024, 640, (1, 16, 1)), ("first tiling 4/4/1", 200, 2048, 320, (1, 4, 4)),
    ("first tiling 8/2/1", 300, 1152, 520, (1, 8, 2)), ("first tiling 16/1/2", 600, 1024, 640, (1, 16, 1 + 2 * 256)),
    ("second tiling 512x128", 1300, 640, 600, (2, 0, 0)), ("second tiling 256x256, 8 workgroups", 1300, 640, 1100, (2, 1, 8 << 8)),
    ("second tiling 256x128 four-wave, 16 workgroups", 1300, 640, 1100, (2, 4, 16 << 8)),
    ("second tiling 128x128", 300, 1024, 520, (2, 5, 0)), ("default dispatch, 2048 tokens", 2048, 512, 4096, None),
]


@pytest.mark.parametrize("label,m,k,n,variant", PATHS)
def test_linear_paths_are_bit_stable(gpu_lib, label, m, k, n, variant):
    w, _, x8, sx = inputs([95, m, k, n], m, k, n)
    packed, scales = B.pack_weights(w, G, B.LAYOUT_TILED)
    for dtype in (torch.float32, torch.bfloat16):
        y = torch.empty((m, n), dtype=dtype, device=DEV)
        if variant is None:
            run = lambda: B.linear(x8, sx, packed, scales, n, G, B.LAYOUT_TILED, out=y)
        else:
            run = lambda: B.linear_variant(x8, sx, packed, scales, n, G, y, *variant)
        repeat_and_compare(f"{label}, {dtype}", run)


def test_other_entry_points_are_bit_stable(gpu_lib):
    m, k, n = 130, 14336, 512
    w, xd, x8, sx = inputs([97], m, k, n)
    packed, scales = B.pack_weights(w, G, B.LAYOUT_TILED)
    ws = torch.empty(B.linear_workspace_bytes(m, k, n, G), dtype=torch.uint8, device=DEV)
    assert ws.numel() > 0
    y = torch.empty((m, n), dtype=torch.bfloat16, device=DEV)
    repeat_and_compare("K ranges across workgroups (workspace)", lambda: B.linear(x8, sx, packed, scales, n, G, B.LAYOUT_TILED, out=y, workspace=ws))
    repeat_and_compare("static workspace", lambda: B.linear_static_workspace(x8, sx, packed, scales, n, G, out=y))
    p2, s2 = B.pack_weights(w, G, B.LAYOUT_TILED, pow2=True)
    repeat_and_compare("power-of-two scales", lambda: B.linear_pow2(x8, sx, p2, s2, n, G, out=y))
    s8 = scales.abs() * 400.0
    w_out = torch.full((n,), 1e-3, dtype=torch.float32, device=DEV)
    repeat_and_compare("two-level", lambda: B.linear_two_level(x8, sx, packed, s8, w_out, n, G, out=y))
    pa, params = B.pack_weights_asym(w, G)
    repeat_and_compare("asymmetric", lambda: B.linear_asym(x8, sx, pa, params, n, G, out=y))
    m1 = 4
    y1 = torch.empty((m1, n), dtype=torch.bfloat16, device=DEV)
    repeat_and_compare("quantization folded in", lambda: B.linear_quantize_in(xd[:m1], sx, packed, scales, n, G, out=y1))
    ys = torch.tensor([0.05], dtype=torch.float32, device=DEV)
    repeat_and_compare("FP8 output", lambda: B.linear_fp8_out(x8, sx, packed, scales, n, G, ys))
