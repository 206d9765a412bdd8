"""Where the floor of the output tolerance comes from: the FP8 matrix unit, not the kernels.

The layer's definition (Sec. 3; Eq. 10, Eq. 4, Eq. 11) fixes the operands exactly, so what separates a kernel's float32
output from the float64 reference is only how the products are added up.  Three checks, on the inputs of the
benchmark configs 1 and 2 and on a hand-made octet:
  - the plain device path (linear_canonical: one float32 FMA per product, no matrix unit) meets the tolerance with the
    tight floor |y - ref| <= 2e-3 * max(|ref|, 1e-3 * A), A the sum of the absolute terms -- kernel logic (operand order,
    scales, rescaling) is exact to float32 rounding;
  - the MFMA paths on the same inputs stay below half of the floor the parity tests use (2e-3 / 64 * A), and are printed;
  - one 16x16x128 MFMA adds the eight products of eight consecutive k after aligning them to the largest of the eight and
    dropping what lies about 14 bits or more below it: a product of 448 * 7 next to seven products of 2^j comes back exact
    for large j and loses the seven small products for small j.  The loss never exceeds 7 * 2^-14 of the largest
    product; it is the same for every kernel that feeds the same operands (they are compared bit for bit elsewhere)."""
import numpy as np
import pytest
import torch

from oracle import w4a8_oracle as o
from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

from test_gpu_parity import dev, host, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TIGHT_FLOOR = 1e-3                    # of A: what plain float32 accumulation meets
PARITY_FLOOR = 2.0 ** -6              # of A: the floor of the parity tests (oracle.within_tolerance's default)


def config_layers():
    """(label, W, X, s_x, group) for config 1 and for the four layer shapes of config 2 at 16 tokens."""
    (m, k, n) = syn.CONFIGS[1]["shapes"][0]
    w, x, s_x = syn.make_layer(1, 0, m, k, n)
    yield "config 1", w, x, s_x, k
    for idx, (k, n) in enumerate(syn.LLAMA3_8B.values()):
        w, x, s_x = syn.make_layer(2, 3 * idx + 2, 16, k, n)
        yield f"config 2, K={k} N={n}, 16 tokens", w, x, s_x, 128


@pytest.mark.parametrize("case", range(5))
def test_plain_fma_path_meets_the_tight_floor_and_mfma_paths_half_the_parity_floor(gpu_lib, case):
    label, w, x, s_x, g = list(config_layers())[case]
    n, k = w.shape
    q, s_w = o.rtn_quantize_weights(w, g)
    x8 = o.quantize_act(x, s_x)
    ref, a = o.linear_ref(x8, s_x, q, s_w, g)
    sx_d, x8_d = dev(np.array([s_x])), dev(x8)
    pc, sc = B.pack_weights(dev(w), g, B.LAYOUT_CANONICAL)
    y_plain = host(B.linear(x8_d, sx_d, pc, sc, n, g, B.LAYOUT_CANONICAL, out_dtype=torch.float32))
    ok, worst = o.within_tolerance(y_plain, ref, a, floor=TIGHT_FLOOR)
    plain_rel = np.max(np.abs(y_plain - ref) / a)
    say(f"  {label}: plain FMA path  worst err/bound (floor 1e-3 A) = {worst:.3e}  max err/A = {plain_rel:.2e}")
    assert ok
    pt, st = B.pack_weights(dev(w), g, B.LAYOUT_TILED)
    y_mfma = host(B.linear(x8_d, sx_d, pt, st, n, g, B.LAYOUT_TILED, out_dtype=torch.float32))
    mfma_rel = np.max(np.abs(y_mfma - ref) / a)
    say(f"  {label}: MFMA path       max err/A = {mfma_rel:.2e}  (parity floor 2e-3/64 = {2e-3 * PARITY_FLOOR:.2e})")
    assert mfma_rel <= 0.5 * 2e-3 * PARITY_FLOOR
    assert plain_rel <= 1e-6


def test_one_mfma_drops_products_far_below_the_largest_of_their_octet(gpu_lib):
    """K = 128, one MFMA per output.  Channel j of the weights multiplies k = 0 by 7 and k = 1..7 by 1; token row t has
    448 at k = 0 and the E4M3 value 2^(t - 9) at k = 1..7 (t = 0..15: 2^-9 .. 2^6), zeros elsewhere.  Exact output:
    3136 + 7 * 2^(t - 9).  All scales are 1, so float32 holds every exact value."""
    m, k, n = 16, 128, 16
    x = np.zeros((m, k), np.float32)
    x[:, 0] = 448.0
    for t in range(m):
        x[t, 1:8] = 2.0 ** (t - 9)
    x8 = o.e4m3_encode(x)
    assert np.array_equal(o.e4m3_decode(x8).astype(np.float32), x)          # all values are on the E4M3 grid
    q = np.zeros((n, k), np.int8)
    q[:, 0] = 7
    q[:, 1:8] = 1
    s_w = np.ones((n, 1), np.float32)
    exact = (3136.0 + 7.0 * 2.0 ** (np.arange(m) - 9.0)).astype(np.float32)
    ref, _ = o.linear_ref(x8, np.float32(1.0), q, s_w, k)
    assert np.array_equal(ref[:, 0].astype(np.float32), exact)
    one = dev(np.array([1.0], np.float32))
    pc, sc = B.pack_weights(dev(q), k, B.LAYOUT_CANONICAL, dev(s_w))
    y_plain = host(B.linear(dev(x8), one, pc, sc, n, k, B.LAYOUT_CANONICAL, out_dtype=torch.float32))
    assert np.array_equal(y_plain[:, 0], exact)                              # plain FMAs: exact
    pt, st = B.pack_weights(dev(q), k, B.LAYOUT_TILED, dev(s_w))
    y_mfma = host(B.linear(dev(x8), one, pt, st, n, k, B.LAYOUT_TILED, out_dtype=torch.float32))
    assert np.array_equal(y_mfma, np.repeat(y_mfma[:, :1], n, axis=1))       # every channel identical
    loss = exact.astype(np.float64) - y_mfma[:, 0].astype(np.float64)
    for t in range(m):
        say(f"  small products 2^{t - 9:+d} (2^{np.log2(3136.0) - (t - 9):.1f} below the largest): exact {exact[t]:.6f}  "
            f"matrix unit {y_mfma[t, 0]:.6f}  lost {loss[t]:.6f} of {7 * 2.0 ** (t - 9):.6f}")
    assert np.all(loss >= 0) and np.all(loss <= 7 * 2.0 ** -14 * 3136.0)     # truncation, never more than the datapath's worst case
    assert np.all(loss[2.0 ** (np.arange(m) - 9.0) >= 3136.0 * 2.0 ** -13] == 0)   # products within 13 bits of the largest: exact
