"""Host-side checks of the C-ABI library: it loads, exports every function the header declares, and rejects bad
arguments before anything is launched (so these run without a GPU; no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2505_14638_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x10000          # a non-NULL, 16-byte aligned dummy address; never dereferenced on the paths tested here


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2505_14638_amd import build
        build.build()
    return B.lib()


def declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("w4a8.h", "w4a8_tuning.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(w4a8_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree(L):
    names = declared_functions()
    assert {"w4a8_quantize_act", "w4a8_pack_weights", "w4a8_linear"} <= set(names)
    for name in names:
        assert hasattr(L, name), f"{name} declared in include/*.h but not exported"
        assert name in B.SIGNATURES, f"{name} has no ctypes signature in the binding"
    assert sorted(B.SIGNATURES) == names


def test_status_strings(L):
    assert B.status_string(0) == "ok"
    seen = {B.status_string(s) for s in range(0, 9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert B.status_string(99) == "unknown status"


def test_sizes(L):
    assert L.w4a8_packed_bytes(1024, 1024, B.LAYOUT_CANONICAL) == 1024 * 512
    assert L.w4a8_packed_bytes(40, 384, B.LAYOUT_TILED) == 48 * 192
    assert L.w4a8_packed_bytes(40, 100, B.LAYOUT_TILED) == 0            # K % 128 != 0
    assert L.w4a8_scales_count(40, 384, 128, B.LAYOUT_TILED) == 48 * 3
    assert L.w4a8_scales_count(40, 384, 384, B.LAYOUT_TILED) == 48
    assert L.w4a8_scales_count(40, 384, 32, B.LAYOUT_CANONICAL) == 40 * 12
    assert L.w4a8_scales_count(40, 384, 32, B.LAYOUT_TILED) == 0        # groups below 128 need the canonical layout
    assert L.w4a8_scales_count(40, 384, 100, B.LAYOUT_CANONICAL) == 0
    assert L.w4a8_linear_workspace_bytes(16, 4096, 4096, 128) == 0


def test_quantize_act_validation(L):
    f = L.w4a8_quantize_act
    assert f(0, B.F32, 4, 64, 64, P, P, 64, None) == 1                  # NULL x
    assert f(P, B.F32, 4, 64, 64, 0, P, 64, None) == 1                  # NULL scale
    assert f(P, 7, 4, 64, 64, P, P, 64, None) == 4                      # dtype
    assert f(P, B.F32, -1, 64, 64, P, P, 64, None) == 2
    assert f(P, B.F32, 4, 64, 32, P, P, 64, None) == 2                  # ldx < K
    assert f(P, B.F32, 4, 64, 64, P, P, 8, None) == 2                   # ldx8 < K
    assert f(P + 2, B.F32, 4, 64, 64, P, P, 64, None) == 6              # misaligned float pointer
    assert f(P, B.F32, 0, 64, 64, P, P, 64, None) == 0                  # M == 0: no-op


def test_act_scale_validation(L):
    f = L.w4a8_act_amax
    assert f(P, B.F32, 0, 64, 64, P, None) == 0
    assert f(0, B.F32, 4, 64, 64, P, None) == 1 and f(P, B.F32, 4, 64, 64, 0, None) == 1
    assert f(P, 9, 4, 64, 64, P, None) == 4 and f(P, B.F32, 4, 64, 32, P, None) == 2
    assert f(P + 2, B.F32, 4, 64, 64, P, None) == 6
    assert L.w4a8_act_scale_from_amax(0, P, None) == 1 and L.w4a8_act_scale_from_amax(P, P + 1, None) == 6


def test_pack_validation(L):
    f = L.w4a8_pack_weights
    assert f(P, B.SRC_F32_RTN, 0, 16, 256, 128, B.LAYOUT_TILED, 0, P, None) == 1
    assert f(P, B.SRC_I8_CODES, 0, 16, 256, 128, B.LAYOUT_TILED, P, P, None) == 1      # codes need scales
    assert f(P, 5, 0, 16, 256, 128, B.LAYOUT_TILED, P, P, None) == 4
    assert f(P, B.SRC_F32_RTN, 0, 16, 256, 100, B.LAYOUT_CANONICAL, P, P, None) == 3   # G does not divide K
    assert f(P, B.SRC_F32_RTN, 0, 16, 256, 64, B.LAYOUT_TILED, P, P, None) == 3        # tiled needs G % 128 == 0
    assert f(P, B.SRC_F32_RTN, 0, 16, 200, 200, B.LAYOUT_TILED, P, P, None) == 5       # tiled needs K % 128 == 0
    assert f(P, B.SRC_F32_RTN, 0, 16, 255, 255, B.LAYOUT_CANONICAL, P, P, None) == 2   # odd K
    assert f(P, B.SRC_F32_RTN, 0, 16, 256, 128, 9, P, P, None) == 5
    assert f(P, B.SRC_F32_RTN, 0, 0, 256, 128, B.LAYOUT_TILED, P, P, None) == 2


def test_linear_validation(L):
    f = L.w4a8_linear
    ok = dict(x8=P, M=4, K=256, ldx8=256, xs=P, packed=P, ws=P, N=64, G=128, layout=B.LAYOUT_TILED, y=P, ydt=B.BF16,
              ldy=64)

    def call(**kw):
        a = {**ok, **kw}
        return f(a["x8"], a["M"], a["K"], a["ldx8"], a["xs"], a["packed"], a["ws"], a["N"], a["G"], a["layout"],
                 a["y"], a["ydt"], a["ldy"], None, 0, None)

    assert call(M=0) == 0
    for key in ("x8", "xs", "packed", "ws", "y"):
        assert call(**{key: 0}) == 1, key
    assert call(M=-3) == 2 and call(N=0) == 2 and call(K=0) == 2
    assert call(ldx8=128) == 2 and call(ldy=32) == 2
    assert call(G=96) == 3 and call(G=64) == 3
    assert call(ydt=3) == 4
    assert call(layout=4) == 5 and call(K=192, ldx8=192, G=192) == 5
    assert call(x8=P + 4) == 6 and call(ldx8=264) == 6 and call(packed=P + 8) == 6
    assert call(y=P + 1) == 6
    assert call(layout=B.LAYOUT_CANONICAL, G=32, M=0) == 0
    # size limits: weights per matrix, groups per matrix, outputs of the canonical layout's layer, strides of the tiled one
    assert call(N=1 << 20, K=1 << 13, ldx8=1 << 13, ldy=1 << 20) == 2                       # 2^33 weights
    assert call(layout=B.LAYOUT_CANONICAL, N=1 << 14, K=1 << 13, ldx8=1 << 13, ldy=1 << 14, G=2) == 2   # 2^26 groups
    assert call(layout=B.LAYOUT_CANONICAL, M=1 << 13, N=1 << 13, ldy=1 << 13, G=32) == 2    # 2^26 canonical outputs
    assert call(ldx8=1 << 23) == 2 and call(ldy=1 << 20) == 2
    # workspace (K ranges across workgroups, Sec. 1: between the two regimes): asked for on few-tile, deep-K shapes only
    wb = L.w4a8_linear_workspace_bytes
    assert wb(8, 14336, 4096, 128) == 0 and wb(8192, 4096, 4096, 128) == 0 and wb(128, 4096, 28672, 128) == 0
    need = wb(128, 14336, 4096, 128)
    assert need > 0 and need % (128 * 4096 * 4) == 0 and need <= 32 << 20     # whole float32 [M, N] planes, one per K range
    assert wb(128, 4096, 4096, 128) == 0 and wb(1024, 14336, 4096, 128) == 0   # shallow K, many tokens: not split
    assert wb(128, 14336, 4096, 96) == 0 and wb(0, 14336, 4096, 128) == 0
    # 41..64 tokens on a deep narrow layer: the few-token kernel without a workspace, K ranges across workgroups with one
    assert wb(40, 14336, 4096, 128) == 0 and wb(48, 14336, 4096, 128) > 0 and wb(64, 4096, 4096, 128) == 0
    assert B.linear_launch_shape(48, 14336, 4096, 128)[0] == 0 and B.linear_launch_shape(48, 14336, 4096, 128, True)[0] == 3
    assert B.linear_launch_shape(64, 4096, 4096, 128)[0] == 0 and B.linear_launch_shape(64, 4096, 6144, 128)[0] == 1
    assert B.linear_launch_shape(48, 4096, 6144, 128)[0] == 0 and B.linear_launch_shape(33, 4096, 28672, 128)[0] == 1
    big = dict(M=128, K=14336, ldx8=14336, N=4096, ldy=4096)

    def call_ws(ws, nbytes, **kw):
        a = {**ok, **big, **kw}
        return f(a["x8"], a["M"], a["K"], a["ldx8"], a["xs"], a["packed"], a["ws"], a["N"], a["G"], a["layout"],
                 a["y"], a["ydt"], a["ldy"], ws, nbytes, None)

    assert call_ws(P, need - 1) == 7 and call_ws(P, 0) == 7                   # too small
    assert call_ws(P + 8, need) == 6                                           # misaligned
    assert call_ws(P, 0, M=0) == 0                                             # nothing needed, nothing launched
    # the variant with its scratch inside the library: same validation, sizes beyond the buffer refused on the host
    fn = L.w4a8_linear_static_workspace
    assert fn(P, 0, 14336, 14336, P, P, P, 4096, 128, P, B.BF16, 4096, None) == 0
    assert fn(0, 128, 14336, 14336, P, P, P, 4096, 128, P, B.BF16, 4096, None) == 1
    assert fn(P, 128, 14336, 14336, P, P, P, 4096, 96, P, B.BF16, 4096, None) == 3
    assert wb(512, 28672, 8192, 128) > 16 << 20
    assert fn(P, 512, 28672, 28672, P, P, P, 8192, 128, P, B.BF16, 8192, None) == 7
    # the launch shape the library chooses, as w4a8_linear_variant takes it
    assert B.linear_launch_shape(1, 4096, 4096, 128) == (0, 1, 16 | (2 << 8), 0)
    assert B.linear_launch_shape(8192, 4096, 4096, 128) == (2, 1, 0, 0) and B.linear_launch_shape(2048, 4096, 4096, 128) == (2, 2, 0, 0) and B.linear_launch_shape(3072, 4096, 6144, 128) == (2, 4, 0, 0)
    assert B.linear_launch_shape(512, 4096, 4096, 128)[0] == 1
    assert B.linear_launch_shape(128, 14336, 4096, 128, True) == (3, 5, 0, 8) and B.linear_launch_shape(128, 14336, 4096, 128)[0] == 1
    assert L.w4a8_linear_launch_shape(128, 14336, 4096, 128, 0, None) == 1 and L.w4a8_linear_launch_shape(0, 14336, 4096, 128, 0, P) == 2
    fs = L.w4a8_linear_splitk_variant
    sk = (P, 128, 14336, 14336, P, P, P, 4096, 128, P, B.BF16, 4096)
    assert fs(*sk, 5, 4, P, 4 * 128 * 4096 * 4 - 1, None) == 7
    assert fs(*sk, 5, 1, P, 1 << 30, None) == 2 and fs(*sk, 5, 113, P, 1 << 30, None) == 2
    assert fs(*sk, 5, 4, None, 1 << 30, None) == 1 and fs(*sk, 5, 4, P + 4, 1 << 30, None) == 6
    fv = L.w4a8_linear_variant
    assert fv(P, 100, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, 1, 1, None) == 2   # skinny path needs M <= 64
    assert fv(P, 4, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 7, 0, 0, None) == 2     # unknown path
    assert fv(P, 0, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, 1, 1, None) == 0


def test_two_level_validation(L):
    f = L.w4a8_linear_two_level
    # x8, M, K, ldx8, xs, packed, s8, s_out, per_channel, N, G, y, ydt, ldy, stream
    assert f(P, 0, 256, 256, P, P, P, P, 1, 64, 128, P, B.BF16, 64, None) == 0         # M == 0: no-op
    assert f(P, 4, 256, 256, P, P, P, 0, 1, 64, 128, P, B.BF16, 64, None) == 1         # NULL output scales
    assert f(P, 4, 256, 256, P, P, 0, P, 1, 64, 128, P, B.BF16, 64, None) == 1         # NULL group scales
    assert f(P, 4, 256, 256, P, P, P, P, 2, 64, 128, P, B.BF16, 64, None) == 4         # per_channel is 0 or 1
    assert f(P, 4, 256, 256, P, P, P, P + 2, 1, 64, 128, P, B.BF16, 64, None) == 6     # misaligned output scales
    assert f(P, 4, 256, 256, P, P, P, P, 1, 64, 96, P, B.BF16, 64, None) == 3          # tiled needs G % 128 == 0
    assert f(P, 4, 200, 200, P, P, P, P, 1, 64, 200, P, B.BF16, 64, None) == 5         # tiled needs K % 128 == 0
    d = L.w4a8_dequant_weights_two_level
    assert d(P, 0, 16, 256, 128, P, None) == 1
    assert d(P, P, 16, 256, 64, P, None) == 3
    assert d(P + 8, P, 16, 256, 128, P, None) == 6


def test_pow2_validation(L):
    f = L.w4a8_linear_pow2
    # x8, M, K, ldx8, xs, packed, scales, N, G, y, ydt, ldy, stream
    assert f(P, 0, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, None) == 0
    assert f(P, 4, 256, 256, P, P, 0, 64, 128, P, B.BF16, 64, None) == 1
    assert f(P, 4, 256, 256, P, P, P, 64, 64, P, B.BF16, 64, None) == 3
    assert f(P, 4, 200, 200, P, P, P, 64, 200, P, B.BF16, 64, None) == 5
    assert f(P, 4, 256, 256, P, P + 4, P, 64, 128, P, B.BF16, 64, None) == 6
    p = L.w4a8_pack_weights
    assert p(P, B.SRC_F32_RTN_POW2, 0, 16, 256, 128, B.LAYOUT_TILED, 0, P, None) == 1
    assert p(P + 2, B.SRC_F32_RTN_POW2, 0, 16, 256, 128, B.LAYOUT_TILED, P, P, None) == 6
    assert p(P, 3, 0, 16, 256, 128, B.LAYOUT_TILED, P, P, None) == 4
    assert L.w4a8_pack_weights_asym(P, B.SRC_F32_RTN_POW2, 0, 0, 16, 256, 128, P, P, None) == 4


def test_asym_validation(L):
    assert L.w4a8_asym_params_bytes(40, 384, 128) == 3 * 3 * 80
    assert L.w4a8_asym_params_bytes(40, 384, 384) == 3 * 80
    assert L.w4a8_asym_params_bytes(40, 384, 64) == 0                   # tiled storage needs G % 128 == 0
    p = L.w4a8_pack_weights_asym
    # src, kind, src_scales, src_zeros, N, K, G, packed, params, stream
    assert p(P, B.SRC_F32_RTN, 0, 0, 16, 256, 128, 0, P, None) == 1
    assert p(P, B.SRC_I8_CODES, P, 0, 16, 256, 128, P, P, None) == 1    # codes need scales and zero-points
    assert p(P, B.SRC_I8_CODES, 0, P, 16, 256, 128, P, P, None) == 1
    assert p(P, 3, 0, 0, 16, 256, 128, P, P, None) == 4
    assert p(P, B.SRC_F32_RTN, 0, 0, 16, 256, 64, P, P, None) == 3
    assert p(P, B.SRC_F32_RTN, 0, 0, 16, 200, 200, P, P, None) == 5
    assert p(P, B.SRC_F32_RTN, 0, 0, 16, 256, 128, P, P + 4, None) == 6 # records are 16-byte aligned
    f = L.w4a8_linear_asym
    # x8, M, K, ldx8, xs, packed, params, N, G, y, ydt, ldy, stream
    assert f(P, 0, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, None) == 0
    assert f(P, 4, 256, 256, P, P, 0, 64, 128, P, B.BF16, 64, None) == 1
    assert f(P, 4, 256, 256, P, P, P + 8, 64, 128, P, B.BF16, 64, None) == 6
    assert f(P, 4, 256, 256, P, P, P, 64, 96, P, B.BF16, 64, None) == 3
    assert f(P, 4, 256, 128, P, P, P, 64, 128, P, B.BF16, 64, None) == 2
    assert f(P, 4, 256, 256, P, P, P, 64, 128, P, 5, 64, None) == 4
    t = L.w4a8_linear_asym_two_level
    # x8, M, K, ldx8, xs, packed, params8, s_out, per_channel, N, G, y, ydt, ldy, stream
    assert t(P, 0, 256, 256, P, P, P, P, 1, 64, 128, P, B.BF16, 64, None) == 0
    assert t(P, 4, 256, 256, P, P, P, 0, 1, 64, 128, P, B.BF16, 64, None) == 1
    assert t(P, 4, 256, 256, P, P, P, P, 3, 64, 128, P, B.BF16, 64, None) == 4
    assert t(P, 4, 256, 256, P, P, P + 4, P, 1, 64, 128, P, B.BF16, 64, None) == 6
    assert L.w4a8_dequant_weights_asym_two_level(P, 0, 16, 256, 128, P, None) == 1
    d = L.w4a8_dequant_weights_asym
    assert d(P, 0, 16, 256, 128, P, None) == 1
    assert d(P, P, 16, 256, 64, P, None) == 3
    assert d(P, P + 8, 16, 256, 128, P, None) == 6


def test_fused_validation(L):
    f = L.w4a8_linear_fp8_out
    # x8, M, K, ldx8, xs, packed, scales, N, G, y_scale, y8, ldy8, stream
    assert f(P, 0, 256, 256, P, P, P, 64, 128, P, P, 64, None) == 0
    assert f(P, 4, 256, 256, P, P, P, 64, 128, 0, P, 64, None) == 1                    # NULL output scale
    assert f(P, 4, 256, 256, P, P, P, 64, 128, P, 0, 64, None) == 1
    assert f(P, 4, 256, 256, P, P, P, 64, 128, P + 2, P, 64, None) == 6
    assert f(P, 4, 256, 256, P, P, P, 64, 128, P, P, 32, None) == 2                    # ldy8 < N
    assert f(P, 4, 256, 256, P, P, P, 64, 96, P, P, 64, None) == 3
    assert L.w4a8_linear(P, 4, 256, 256, P, P, P, 64, 128, B.LAYOUT_TILED, P, 2, 64, None, 0, None) == 4   # 2 is not public
    g = L.w4a8_linear_silu_mul_fp8_out
    # x8, M, K, ldx8, xs, packed, scales, F, G, h_scale, h8, ldh8, stream
    assert g(P, 0, 256, 256, P, P, P, 64, 128, P, P, 64, None) == 0
    assert g(P, 4, 256, 256, P, P, P, 40, 128, P, P, 64, None) == 2                    # F % 16 != 0
    assert g(P, 4, 256, 256, P, P, P, 64, 128, P, P, 32, None) == 2                    # ldh8 < F
    assert g(P, 4, 256, 256, P, P, P, 64, 128, 0, P, 64, None) == 1
    q = L.w4a8_silu_mul_quantize
    assert q(P, 0, 64, 128, P, P, 64, None) == 0
    assert q(P, 4, 64, 64, P, P, 64, None) == 2                                        # ldgu < 2F
    assert q(P, 4, 64, 128, 0, P, 64, None) == 1
    assert q(P, 4, 64, 128, P, P, 32, None) == 2


def test_linear_quantize_in_validation(L):
    f = L.w4a8_linear_quantize_in
    # x, x_dtype, M, K, ldx, x_scale, packed, w_scales, N, G, y, y_dtype, ldy, x8_out, stream
    assert f(P, B.F32, 0, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 0
    assert f(P, B.F32, 17, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 2              # more than 16 tokens
    assert f(P, B.F32, 16, 8192, 8192, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 2            # M * K > 65536
    assert f(P, B.F32, 4, 256, 128, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 2               # ldx < K
    assert f(P, B.F32, 4, 256, 258, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 6               # ldx not a multiple of 4
    assert f(P, B.BF16, 4, 256, 260, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 6              # ... of 8 for bf16
    assert f(P + 4, B.F32, 4, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 6
    assert f(P, B.F32, 4, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, P + 8, None) == 6
    assert f(0, B.F32, 4, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 1
    assert f(P, 7, 4, 256, 256, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 4
    assert f(P, B.F32, 4, 200, 200, P, P, P, 64, 128, P, B.BF16, 64, 0, None) == 5
    assert f(P, B.F32, 4, 256, 256, P, P, P, 64, 96, P, B.BF16, 64, 0, None) == 3


def test_few_token_forms_split_k_alike(L):
    """The fused forms of the few-token kernel are byte-identical to the sequences they replace only if they add up the
    same partial sums in the same order, i.e. split K over the same number of wavefronts as the plain layer on the same
    (M, K, N).  Checked on the host over a grid of sizes (the launch-shape function launches nothing)."""
    assert L.w4a8_linear_few_token_shape(1, 4096, 4096, 128, 0, None) == 1
    assert L.w4a8_linear_few_token_shape(65, 4096, 4096, 128, 0, P) == 2 and L.w4a8_linear_few_token_shape(1, 4096, 4096, 128, 5, P) == 2
    assert L.w4a8_linear_few_token_shape(17, 1024, 4096, 128, 3, P) == 2 and L.w4a8_linear_few_token_shape(1, 4096, 4080, 128, 2, P) == 2
    assert B.linear_few_token_shape(1, 8192, 8192, 128) == (1, 8, 4) and B.linear_few_token_shape(1, 8192, 8192, 128, "fp8_out") == (1, 8, 2)
    assert B.linear_few_token_shape(16, 8192, 10240, 128) == (4, 8, 2) and B.linear_few_token_shape(1, 4096, 6144, 128) == (2, 16, 2)
    checked = 0
    for k in (128, 512, 1024, 4096, 8192, 14336, 28672):
        for n in (32, 96, 2048, 4096, 6144, 8192, 10240, 16384, 28672, 57344, 128256):
            if (n + 15) // 16 * 16 * k > 1 << 32:
                continue
            for m in (1, 2, 4, 7, 8, 9, 15, 16, 17, 24, 32, 33, 48, 64):
                nt, waves, depth = B.linear_few_token_shape(m, k, n, 128)
                assert nt in (1, 2, 4) and 1 <= waves <= 16 and depth in (2, 4)
                assert B.linear_few_token_shape(m, k, n, 128, "fp8_out")[1] == waves
                if n % 32 == 0:
                    nt_s, waves_s, _ = B.linear_few_token_shape(m, k, n, 128, "silu_mul_fp8_out")
                    assert waves_s == waves and nt_s % 2 == 0
                if m <= 16 and m * k <= 65536:
                    for form in ("quantize_in", "quantize_in_fp8_out"):
                        nt_q, waves_q, depth_q = B.linear_few_token_shape(m, k, n, 128, form)
                        assert waves_q == waves and nt_q <= 2 and depth_q == 2
                checked += 1
    assert checked > 900


def test_launch_shape_is_built_and_consistent_for_every_size(L):
    """w4a8_linear's own choice over a grid of sizes: always a built combination (never W4A8_ERR_SHAPE for valid sizes),
    K ranges across workgroups exactly where w4a8_linear_workspace_bytes() asks for a workspace, and the same launch with
    and without a workspace everywhere else."""
    second_tiling_tiles = {0, 1, 2, 3, 4, 5}
    first_tiling = {(16, 1, 1), (8, 1, 1), (8, 2, 1), (4, 1, 1), (4, 2, 1), (4, 4, 1), (16, 1, 2)}
    n_checked = 0
    for k in (128, 1024, 4096, 8192, 14336, 28672):
        for n in (16, 100, 4096, 6144, 10240, 28672, 57344):
            for m in (1, 16, 17, 32, 33, 40, 41, 48, 49, 64, 65, 100, 128, 192, 256, 300, 512, 640, 1000, 2048, 3072, 8192, 20000):
                plain = B.linear_launch_shape(m, k, n, 128)
                with_ws = B.linear_launch_shape(m, k, n, 128, True)
                need = L.w4a8_linear_workspace_bytes(m, k, n, 128)
                for path, p0, p1, ranges in (plain, with_ws):
                    assert path in (0, 1, 2, 3)
                    if path == 0:
                        assert m <= 64 and p0 in (1, 2, 4) and 1 <= (p1 & 0xFF) <= 16 and (p1 >> 8) in (2, 4)
                    elif path == 1:
                        assert (p0, p1 & 0xFF, p1 >> 8) in first_tiling
                    else:
                        assert p0 in second_tiling_tiles
                    assert (ranges >= 2) == (path == 3) and (path != 3 or ranges <= k // 128)
                assert plain[0] != 3 and (with_ws[0] == 3) == (need > 0)
                if need == 0:
                    assert with_ws == plain
                else:
                    assert need == with_ws[3] * m * ((n + 63) // 64 * 64) * 4
                n_checked += 1
    assert n_checked == 6 * 7 * 23


def test_linear_quantize_in_fp8_out_validation(L):
    f = L.w4a8_linear_quantize_in_fp8_out
    # x, x_dtype, M, K, ldx, x_scale, packed, w_scales, N, G, y_scale, y8, ldy8, x8_out, stream
    assert f(P, B.BF16, 0, 256, 256, P, P, P, 64, 128, P, P, 64, 0, None) == 0
    assert f(P, B.BF16, 17, 256, 256, P, P, P, 64, 128, P, P, 64, 0, None) == 2                  # more than 16 tokens
    assert f(P, B.BF16, 16, 8192, 8192, P, P, P, 64, 128, P, P, 64, 0, None) == 2                # M * K > 65536
    assert f(P, B.BF16, 4, 256, 128, P, P, P, 64, 128, P, P, 64, 0, None) == 2                   # ldx < K
    assert f(P, B.BF16, 4, 256, 256, P, P, P, 64, 128, P, P, 32, 0, None) == 2                   # ldy8 < N
    assert f(P, B.BF16, 4, 256, 260, P, P, P, 64, 128, P, P, 64, 0, None) == 6
    assert f(P, B.BF16, 4, 256, 256, P, P, P, 64, 128, P + 2, P, 64, 0, None) == 6               # y_scale not 4-byte aligned
    assert f(P, B.BF16, 4, 256, 256, P, P, P, 64, 128, P, P, 64, P + 8, None) == 6
    assert f(P, B.BF16, 4, 256, 256, P, P, P, 64, 128, 0, P, 64, 0, None) == 1                   # no output scale
    assert f(P, B.BF16, 4, 256, 256, P, P, P, 64, 128, P, 0, 64, 0, None) == 1
    assert f(P, 7, 4, 256, 256, P, P, P, 64, 128, P, P, 64, 0, None) == 4
    assert f(P, B.BF16, 4, 200, 200, P, P, P, 64, 128, P, P, 64, 0, None) == 5
    assert f(P, B.BF16, 4, 256, 256, P, P, P, 64, 96, P, P, 64, 0, None) == 3


def test_calibration_validation(L):
    ha = L.w4a8_hessian_accumulate
    assert ha(P, B.F32, 0, 64, 64, P, None) == 0
    assert ha(0, B.F32, 4, 64, 64, P, None) == 1 and ha(P, B.F32, 4, 64, 32, P, None) == 2 and ha(P, 5, 4, 64, 64, P, None) == 4
    gp = L.w4a8_gar_permutation
    assert gp(0, 256, 128, P, None) == 1 and gp(P, 256, 128, 0, None) == 1
    assert gp(P, 200, 200, P, None) == 5 and gp(P, 256, 64, P, None) == 3
    assert L.w4a8_dpq_workspace_bytes(10, 256) == (10 * 256 + 10 * 128) * 4
    hf = L.w4a8_hessian_inverse_factor
    nb = L.w4a8_hessian_factor_workspace_bytes(256)
    assert nb == (2 * 256 * 256 + 256 * 64 + 2) * 8 and L.w4a8_hessian_factor_workspace_bytes(200) == 0
    # h, K, damp, perm, workspace, bytes, u, info, stream
    assert hf(0, 256, 0.01, 0, P, nb, P, P, None) == 1 and hf(P, 256, 0.01, 0, P, nb, P, 0, None) == 1
    assert hf(P, 200, 0.01, 0, P, nb, P, P, None) == 2 and hf(P, 256, -1.0, 0, P, nb, P, P, None) == 2
    assert hf(P, 256, float("nan"), 0, P, nb, P, P, None) == 2
    assert hf(P, 256, 0.01, P + 2, P, nb, P, P, None) == 6 and hf(P, 256, 0.01, 0, P + 8, nb, P, P, None) == 6
    assert hf(P, 256, 0.01, 0, P, nb - 1, P, P, None) == 7
    f = L.w4a8_dpq_calibrate
    # w, u, s_w, per_channel, perm, N, K, G, codes, scales, zeros, workspace, bytes, stream
    ok = L.w4a8_dpq_workspace_bytes(16, 256)
    assert f(0, P, P, 1, 0, 16, 256, 128, P, P, P, P, ok, None) == 1
    assert f(P, P, P, 1, 0, 16, 256, 128, P, P, P, 0, ok, None) == 1
    assert f(P, P, P, 2, 0, 16, 256, 128, P, P, P, P, ok, None) == 4
    assert f(P, P, P, 1, 0, 16, 256, 96, P, P, P, P, ok, None) == 3
    assert f(P, P, P, 1, 0, 16, 200, 200, P, P, P, P, ok, None) == 5
    assert f(P, P, P, 1, P + 2, 16, 256, 128, P, P, P, P, ok, None) == 6
    assert f(P, P, P, 1, 0, 16, 256, 128, P, P, P, P, ok - 1, None) == 7
    fm = L.w4a8_dpq_calibrate_mse
    # w, u, s_w, per_channel, perm, N, K, G, mse_grid, mse_max_shrink, codes, scales, zeros, workspace, bytes, stream
    assert fm(P, P, P, 1, 0, 16, 256, 128, 20, 0.8, P, P, P, P, ok - 1, None) == 7
    assert fm(P, P, P, 1, 0, 16, 256, 128, -1, 0.8, P, P, P, P, ok, None) == 2
    assert fm(P, P, P, 1, 0, 16, 256, 128, 2000, 0.8, P, P, P, P, ok, None) == 2
    assert fm(P, P, P, 1, 0, 16, 256, 128, 20, 1.0, P, P, P, P, ok, None) == 2
    assert fm(P, P, P, 1, 0, 16, 256, 128, 20, float("nan"), P, P, P, P, ok, None) == 2
    assert fm(0, P, P, 1, 0, 16, 256, 128, 20, 0.5, P, P, P, P, ok, None) == 1


def test_other_validation(L):
    assert L.w4a8_dequant_weights(0, 16, 256, B.LAYOUT_TILED, P, None) == 1
    assert L.w4a8_dequant_weights(P, 16, 200, B.LAYOUT_TILED, P, None) == 5
    assert L.w4a8_silu_mul(P, 4, 64, 64, P, 64, None) == 2              # ldgu < 2F
    assert L.w4a8_silu_mul(0, 4, 64, 128, P, 64, None) == 1
    assert L.w4a8_silu_mul(P, 0, 64, 128, P, 64, None) == 0


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_interleave_gate_up_row_order():
    """The row order the fused gate|up layer expects: bands of 16 gate rows followed by the 16 up rows of the same
    channels (host-side re-ordering; runs on CPU tensors)."""
    import torch
    f, k = 48, 8
    w = torch.arange(2 * f * k, dtype=torch.float32).reshape(2 * f, k)
    wi = B.interleave_gate_up(w)
    assert wi.shape == w.shape
    for p in range(f // 16):
        for i in range(16):
            assert torch.equal(wi[32 * p + i], w[16 * p + i])               # gate row 16p + i
            assert torch.equal(wi[32 * p + 16 + i], w[f + 16 * p + i])      # up row 16p + i
