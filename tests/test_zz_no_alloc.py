"""w4a8_linear_static_workspace (the layer for callers that cannot allocate: its scratch lives inside the library) against
w4a8_linear with a caller's workspace, through the C-ABI: identical bytes, on two calls in a row of which the second is
smaller (the scratch keeps the first call's contents), and on a shape that needs no scratch; sizes beyond the buffer
are refused."""
import numpy as np
import pytest
import torch

from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
G = 128


def layer(seed, m, k, n):
    rng = np.random.default_rng(seed)
    w = torch.from_numpy(syn.make_weights(rng, n, k)).to(DEV)
    packed, scales = B.pack_weights(w, G, B.LAYOUT_TILED)
    x = syn.make_activations(rng, m, k, 0.01, 20.0)
    sx = torch.tensor([syn.static_act_scale(x)], dtype=torch.float32, device=DEV)
    x8 = B.quantize_act(torch.from_numpy(x).to(DEV), sx)
    return x8, sx, packed, scales


def test_static_workspace_matches_the_caller_workspace(gpu_lib):
    k, n = 14336, 1024
    limit = 16 << 20
    for m, dtype in ((200, torch.float32), (96, torch.bfloat16), (70, torch.float32)):   # the later calls are smaller
        need = B.linear_workspace_bytes(m, k, n, G)
        assert 0 < need <= limit, (m, need)
        print(f"static workspace: M={m} K={k} N={n} needs {need} bytes", flush=True)
        x8, sx, packed, scales = layer([91, m], m, k, n)
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        want = B.linear(x8, sx, packed, scales, n, G, B.LAYOUT_TILED, out_dtype=dtype, workspace=ws)
        got = B.linear_static_workspace(x8, sx, packed, scales, n, G, out_dtype=dtype)
        torch.cuda.synchronize()
        view = torch.int32 if dtype == torch.float32 else torch.int16
        assert torch.equal(got.view(view), want.view(view)), (m, dtype)
        assert torch.isfinite(got.float()).all()
    # a shape that takes no scratch goes straight through
    x8, sx, packed, scales = layer([93], 8, 1024, 256)
    assert B.linear_workspace_bytes(8, 1024, 256, G) == 0
    a = B.linear_static_workspace(x8, sx, packed, scales, 256, G, out_dtype=torch.float32)
    b = B.linear(x8, sx, packed, scales, 256, G, B.LAYOUT_TILED, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_static_workspace_refuses_what_does_not_fit(gpu_lib):
    m, k, n = 512, 28672, 8192                                   # Llama-3-70B down projection at 512 tokens: 32 MiB of partial sums
    need = B.linear_workspace_bytes(m, k, n, G)
    assert need > 16 << 20
    x8 = torch.zeros((m, k), dtype=torch.uint8, device=DEV)
    sx = torch.ones(1, dtype=torch.float32, device=DEV)
    packed = torch.zeros(n * k // 2, dtype=torch.uint8, device=DEV)
    scales = torch.ones(n * k // G, dtype=torch.float32, device=DEV)
    with pytest.raises(B.W4A8Error) as e:
        B.linear_static_workspace(x8, sx, packed, scales, n, G)
    assert e.value.status == 7
