"""Thin ctypes binding of libw4a8.so: same entry-point names as include/w4a8.h, argument marshalling only.

PyTorch supplies device memory (`tensor.data_ptr()`) and the current stream; every computation happens in the
library's kernels.  There is no CPU or eager fallback: `lib()` raises if the library has not been built, and every
wrapper raises `W4A8Error` on a non-zero status.
"""
from __future__ import annotations

import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libw4a8.so")

# enums of include/w4a8.h
F32, BF16 = 0, 1
SRC_F32_RTN, SRC_I8_CODES, SRC_F32_RTN_POW2 = 0, 1, 2
LAYOUT_CANONICAL, LAYOUT_TILED = 0, 1

_c_i64, _c_i32, _c_vp, _c_sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t

SIGNATURES = {
    "w4a8_packed_bytes": (_c_sz, [_c_i64, _c_i64, _c_i32]),
    "w4a8_scales_count": (_c_sz, [_c_i64, _c_i64, _c_i32, _c_i32]),
    "w4a8_quantize_act": (_c_i32, [_c_vp, _c_i32, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_i64, _c_vp]),
    "w4a8_act_amax": (_c_i32, [_c_vp, _c_i32, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp]),
    "w4a8_act_scale_from_amax": (_c_i32, [_c_vp, _c_vp, _c_vp]),
    "w4a8_pack_weights": (_c_i32, [_c_vp, _c_i32, _c_vp, _c_i64, _c_i64, _c_i32, _c_i32, _c_vp, _c_vp, _c_vp]),
    "w4a8_linear_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_i64, _c_i32]),
    "w4a8_linear": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_i32, _c_vp,
                             _c_i32, _c_i64, _c_vp, _c_sz, _c_vp]),
    "w4a8_linear_static_workspace": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp,
                                              _c_i32, _c_i64, _c_vp]),
    "w4a8_linear_variant": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp,
                                     _c_i32, _c_i64, _c_i32, _c_i32, _c_i32, _c_vp]),
    "w4a8_linear_launch_shape": (_c_i32, [_c_i64, _c_i64, _c_i64, _c_i32, _c_i32, _c_vp]),
    "w4a8_linear_few_token_shape": (_c_i32, [_c_i64, _c_i64, _c_i64, _c_i32, _c_i32, _c_vp]),
    "w4a8_linear_splitk_variant": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp,
                                            _c_i32, _c_i64, _c_i32, _c_i32, _c_vp, _c_sz, _c_vp]),
    "w4a8_dequant_weights": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i32, _c_vp, _c_vp]),
    "w4a8_linear_two_level": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_vp, _c_i32, _c_i64, _c_i32,
                                       _c_vp, _c_i32, _c_i64, _c_vp]),
    "w4a8_linear_two_level_variant": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_vp, _c_i32, _c_i64,
                                               _c_i32, _c_vp, _c_i32, _c_i64, _c_i32, _c_i32, _c_vp]),
    "w4a8_dequant_weights_two_level": (_c_i32, [_c_vp, _c_vp, _c_i64, _c_i64, _c_i32, _c_vp, _c_vp]),
    "w4a8_linear_pow2": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp, _c_i32,
                                  _c_i64, _c_vp]),
    "w4a8_asym_params_bytes": (_c_sz, [_c_i64, _c_i64, _c_i32]),
    "w4a8_pack_weights_asym": (_c_i32, [_c_vp, _c_i32, _c_vp, _c_vp, _c_i64, _c_i64, _c_i32, _c_vp, _c_vp, _c_vp]),
    "w4a8_linear_asym": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp, _c_i32,
                                  _c_i64, _c_vp]),
    "w4a8_dequant_weights_asym": (_c_i32, [_c_vp, _c_vp, _c_i64, _c_i64, _c_i32, _c_vp, _c_vp]),
    "w4a8_linear_asym_two_level": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_vp, _c_i32, _c_i64,
                                            _c_i32, _c_vp, _c_i32, _c_i64, _c_vp]),
    "w4a8_dequant_weights_asym_two_level": (_c_i32, [_c_vp, _c_vp, _c_i64, _c_i64, _c_i32, _c_vp, _c_vp]),
    "w4a8_hessian_accumulate": (_c_i32, [_c_vp, _c_i32, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp]),
    "w4a8_gar_permutation": (_c_i32, [_c_vp, _c_i64, _c_i32, _c_vp, _c_vp]),
    "w4a8_dpq_workspace_bytes": (_c_sz, [_c_i64, _c_i64]),
    "w4a8_hessian_factor_workspace_bytes": (_c_sz, [_c_i64]),
    "w4a8_hessian_inverse_factor": (_c_i32, [_c_vp, _c_i64, ctypes.c_double, _c_vp, _c_vp, _c_sz, _c_vp, _c_vp, _c_vp]),
    "w4a8_dpq_calibrate": (_c_i32, [_c_vp, _c_vp, _c_vp, _c_i32, _c_vp, _c_i64, _c_i64, _c_i32, _c_vp, _c_vp, _c_vp, _c_vp,
                                    _c_sz, _c_vp]),
    "w4a8_dpq_calibrate_mse": (_c_i32, [_c_vp, _c_vp, _c_vp, _c_i32, _c_vp, _c_i64, _c_i64, _c_i32, _c_i32, ctypes.c_float,
                                        _c_vp, _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "w4a8_linear_quantize_in": (_c_i32, [_c_vp, _c_i32, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp,
                                         _c_i32, _c_i64, _c_vp, _c_vp]),
    "w4a8_linear_quantize_in_fp8_out": (_c_i32, [_c_vp, _c_i32, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32,
                                                 _c_vp, _c_vp, _c_i64, _c_vp, _c_vp]),
    "w4a8_silu_mul": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_i64, _c_vp]),
    "w4a8_linear_fp8_out": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp, _c_vp,
                                     _c_i64, _c_vp]),
    "w4a8_linear_silu_mul_fp8_out": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_vp, _c_i64, _c_i32, _c_vp,
                                              _c_vp, _c_i64, _c_vp]),
    "w4a8_silu_mul_quantize": (_c_i32, [_c_vp, _c_i64, _c_i64, _c_i64, _c_vp, _c_vp, _c_i64, _c_vp]),
    "w4a8_probe_stream_read": (_c_i32, [_c_vp, _c_sz, _c_vp, _c_vp]),
    "w4a8_probe_mfma_e4m3": (_c_i32, [_c_i32, _c_vp, _c_vp]),
    "w4a8_probe_mfma_flop": (ctypes.c_double, [_c_i32]),
    "w4a8_status_string": (ctypes.c_char_p, [_c_i32]),
}

_lib = None


class W4A8Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def lib() -> ctypes.CDLL:
    """Load libw4a8.so (built by paper_2505_14638_amd.build); no fallback when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2505_14638_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def status_string(status: int) -> str:
    return lib().w4a8_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise W4A8Error(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def packed_bytes(n: int, k: int, layout: int) -> int:
    return lib().w4a8_packed_bytes(n, k, layout)


def scales_count(n: int, k: int, group_size: int, layout: int) -> int:
    return lib().w4a8_scales_count(n, k, group_size, layout)


def quantize_act(x: torch.Tensor, scale: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """x [M, K] float32/bf16 (row stride free), scale: 1-element float32 device tensor -> uint8 [M, K]."""
    m, k = x.shape
    assert x.stride(1) == 1 and scale.dtype == torch.float32
    if out is None:
        out = torch.empty((m, k), dtype=torch.uint8, device=x.device)
    _check(lib().w4a8_quantize_act(x.data_ptr(), _dtype_code(x), m, k, x.stride(0) if m > 1 else max(k, x.stride(0)),
                                   scale.data_ptr(), out.data_ptr(), out.stride(0) if m > 1 else max(k, out.stride(0)),
                                   _stream()), "w4a8_quantize_act")
    return out


def calibrate_act_scale(batches) -> torch.Tensor:
    """Static activation scale (Eq. 13) over an iterable of [M, K] float32/bf16 device tensors: max|X| / 448."""
    amax = scale = None
    for x in batches:
        if amax is None:
            amax = torch.zeros(1, dtype=torch.float32, device=x.device)
            scale = torch.empty(1, dtype=torch.float32, device=x.device)
        m, k = x.shape
        assert x.stride(1) == 1
        _check(lib().w4a8_act_amax(x.data_ptr(), _dtype_code(x), m, k, x.stride(0) if m > 1 else max(k, x.stride(0)),
                                   amax.data_ptr(), _stream()), "w4a8_act_amax")
    _check(lib().w4a8_act_scale_from_amax(amax.data_ptr(), scale.data_ptr(), _stream()), "w4a8_act_scale_from_amax")
    return scale


def pack_weights(src: torch.Tensor, group_size: int, layout: int, src_scales: torch.Tensor | None = None,
                 pow2: bool = False):
    """src: float32 W [N, K] (round-to-nearest inside the library; pow2: with power-of-two scales) or int8 codes
    [N, K] with src_scales [N, K/group_size].  Returns (packed uint8 1-D, scales float32 1-D) in `layout`."""
    n, k = src.shape
    assert src.is_contiguous()
    kind = (SRC_F32_RTN_POW2 if pow2 else SRC_F32_RTN) if src.dtype == torch.float32 else SRC_I8_CODES
    nbytes, nscales = packed_bytes(n, k, layout), scales_count(n, k, group_size, layout)
    packed = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=src.device)
    scales = torch.empty(max(nscales, 1), dtype=torch.float32, device=src.device)
    sp = 0
    if kind == SRC_I8_CODES:
        assert src.dtype == torch.int8 and src_scales is not None and src_scales.is_contiguous()
        sp = src_scales.data_ptr()
    _check(lib().w4a8_pack_weights(src.data_ptr(), kind, sp, n, k, group_size, layout, packed.data_ptr(),
                                   scales.data_ptr(), _stream()), "w4a8_pack_weights")
    return packed[:nbytes], scales[:nscales]


def linear_workspace_bytes(m: int, k: int, n: int, group_size: int) -> int:
    return lib().w4a8_linear_workspace_bytes(m, k, n, group_size)


def linear(x8: torch.Tensor, x_scale: torch.Tensor, packed: torch.Tensor, w_scales: torch.Tensor, n: int,
           group_size: int, layout: int, out_dtype: torch.dtype = torch.bfloat16,
           out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """w4a8_linear; `workspace`: a uint8 device tensor of at least linear_workspace_bytes(m, k, n, group_size) bytes, or
    None to run without scratch."""
    m, k = x8.shape
    assert x8.dtype == torch.uint8 and x8.stride(1) == 1
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x8.device)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (0, 0)
    _check(lib().w4a8_linear(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)), x_scale.data_ptr(),
                             packed.data_ptr(), w_scales.data_ptr(), n, group_size, layout, out.data_ptr(),
                             _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)), ws_ptr, ws_bytes,
                             _stream()), "w4a8_linear")
    return out


def linear_static_workspace(x8, x_scale, packed, w_scales, n, group_size, out_dtype=torch.bfloat16, out=None):
    """w4a8_linear_static_workspace: the layer with its scratch inside the library (no allocation by the call)."""
    m, k = x8.shape
    assert x8.dtype == torch.uint8 and x8.stride(1) == 1
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x8.device)
    _check(lib().w4a8_linear_static_workspace(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                              x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), n, group_size,
                                              out.data_ptr(), _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)),
                                              _stream()), "w4a8_linear_static_workspace")
    return out


def linear_launch_shape(m: int, k: int, n: int, group_size: int, with_workspace: bool = False):
    """(path, param0, param1, k_ranges) of the launch w4a8_linear chooses for these sizes (see w4a8_linear_variant)."""
    out = (ctypes.c_int32 * 4)()
    _check(lib().w4a8_linear_launch_shape(m, k, n, group_size, 1 if with_workspace else 0, ctypes.addressof(out)),
           "w4a8_linear_launch_shape")
    return tuple(int(v) for v in out)


FEW_TOKEN_FORMS = {"linear": 0, "fp8_out": 1, "silu_mul_fp8_out": 2, "quantize_in": 3, "quantize_in_fp8_out": 4}


def linear_few_token_shape(m: int, k: int, n: int, group_size: int, form: str = "linear"):
    """(bands per wavefront, wavefronts per workgroup = split of K, chunks in flight) of the few-token kernel for a form."""
    out = (ctypes.c_int32 * 3)()
    _check(lib().w4a8_linear_few_token_shape(m, k, n, group_size, FEW_TOKEN_FORMS[form], ctypes.addressof(out)),
           "w4a8_linear_few_token_shape")
    return tuple(int(v) for v in out)


def linear_splitk_variant(x8, x_scale, packed, w_scales, n, group_size, out, tile: int, ksplit: int, workspace: torch.Tensor):
    m, k = x8.shape
    _check(lib().w4a8_linear_splitk_variant(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                            x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), n, group_size,
                                            out.data_ptr(), _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)),
                                            tile, ksplit, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                            _stream()), "w4a8_linear_splitk_variant")
    return out


def linear_quantize_in(x, x_scale, packed, w_scales, n, group_size, out=None, out_dtype=torch.bfloat16, x8_out=None):
    """w4a8_linear_quantize_in: activations x float32/bf16 [M, K] (M <= 16, M * K <= 65536), quantized inside the layer."""
    m, k = x.shape
    assert x.stride(1) == 1
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x.device)
    assert x8_out is None or (x8_out.dtype == torch.uint8 and x8_out.is_contiguous() and tuple(x8_out.shape) == (m, k))
    _check(lib().w4a8_linear_quantize_in(x.data_ptr(), _dtype_code(x), m, k, x.stride(0) if m > 1 else max(k, x.stride(0)),
                                         x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), n, group_size,
                                         out.data_ptr(), _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)),
                                         x8_out.data_ptr() if x8_out is not None else None, _stream()),
           "w4a8_linear_quantize_in")
    return out


def linear_quantize_in_fp8_out(x, x_scale, packed, w_scales, n, group_size, y_scale, out=None, x8_out=None):
    """w4a8_linear_quantize_in_fp8_out: x float32/bf16 [M, K] quantized inside the layer, output E4M3 bytes [M, N] for the next layer."""
    m, k = x.shape
    assert x.stride(1) == 1
    if out is None:
        out = torch.empty((m, n), dtype=torch.uint8, device=x.device)
    assert out.dtype == torch.uint8 and out.stride(1) == 1
    assert x8_out is None or (x8_out.dtype == torch.uint8 and x8_out.is_contiguous() and tuple(x8_out.shape) == (m, k))
    _check(lib().w4a8_linear_quantize_in_fp8_out(x.data_ptr(), _dtype_code(x), m, k, x.stride(0) if m > 1 else max(k, x.stride(0)),
                                                 x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), n, group_size,
                                                 y_scale.data_ptr(), out.data_ptr(),
                                                 out.stride(0) if m > 1 else max(n, out.stride(0)),
                                                 x8_out.data_ptr() if x8_out is not None else None, _stream()),
           "w4a8_linear_quantize_in_fp8_out")
    return out


def linear_variant(x8, x_scale, packed, w_scales, n, group_size, out, path: int, param0: int, param1: int):
    m, k = x8.shape
    _check(lib().w4a8_linear_variant(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                     x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), n, group_size,
                                     out.data_ptr(), _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)),
                                     path, param0, param1, _stream()), "w4a8_linear_variant")
    return out


def linear_two_level_variant(x8, x_scale, packed, w_scales8, w_out_scales, n, group_size, out, tile: int, param1: int = 0):
    """w4a8_linear_two_level_variant: the two-level layer on a chosen tile of the second tiling."""
    m, k = x8.shape
    per_channel = 1 if w_out_scales.numel() > 1 else 0
    assert w_out_scales.numel() in (1, n) and w_out_scales.dtype == torch.float32
    _check(lib().w4a8_linear_two_level_variant(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                               x_scale.data_ptr(), packed.data_ptr(), w_scales8.data_ptr(),
                                               w_out_scales.data_ptr(), per_channel, n, group_size, out.data_ptr(),
                                               _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)),
                                               tile, param1, _stream()), "w4a8_linear_two_level_variant")
    return out


def linear_two_level(x8, x_scale, packed, w_scales8, w_out_scales, n, group_size, out=None, out_dtype=torch.bfloat16):
    """w4a8_linear_two_level; `w_out_scales` holds N floats (per channel) or one (per tensor)."""
    m, k = x8.shape
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x8.device)
    per_channel = 1 if w_out_scales.numel() > 1 else 0
    assert w_out_scales.numel() in (1, n) and w_out_scales.dtype == torch.float32
    _check(lib().w4a8_linear_two_level(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                       x_scale.data_ptr(), packed.data_ptr(), w_scales8.data_ptr(),
                                       w_out_scales.data_ptr(), per_channel, n, group_size, out.data_ptr(),
                                       _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)), _stream()),
           "w4a8_linear_two_level")
    return out


def dequant_weights_two_level(packed: torch.Tensor, w_scales8: torch.Tensor, n: int, k: int, group_size: int) -> torch.Tensor:
    w8 = torch.empty((n, k), dtype=torch.uint8, device=packed.device)
    _check(lib().w4a8_dequant_weights_two_level(packed.data_ptr(), w_scales8.data_ptr(), n, k, group_size, w8.data_ptr(),
                                                _stream()), "w4a8_dequant_weights_two_level")
    return w8


def linear_pow2(x8, x_scale, packed, w_scales, n, group_size, out=None, out_dtype=torch.bfloat16):
    m, k = x8.shape
    assert x8.dtype == torch.uint8 and x8.stride(1) == 1
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x8.device)
    _check(lib().w4a8_linear_pow2(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)), x_scale.data_ptr(),
                                  packed.data_ptr(), w_scales.data_ptr(), n, group_size, out.data_ptr(), _dtype_code(out),
                                  out.stride(0) if m > 1 else max(n, out.stride(0)), _stream()), "w4a8_linear_pow2")
    return out


def asym_params_bytes(n: int, k: int, group_size: int) -> int:
    return lib().w4a8_asym_params_bytes(n, k, group_size)


def pack_weights_asym(src: torch.Tensor, group_size: int, src_scales: torch.Tensor | None = None,
                      src_zeros: torch.Tensor | None = None):
    """Asymmetric format.  src: float32 W [N, K] (quantized inside the library) or uint8 codes [N, K] with src_scales
    float32 and src_zeros uint8, both [N, K/group_size].  Returns (packed uint8 1-D, params uint8 1-D)."""
    n, k = src.shape
    assert src.is_contiguous()
    kind = SRC_F32_RTN if src.dtype == torch.float32 else SRC_I8_CODES
    nbytes, nparams = packed_bytes(n, k, LAYOUT_TILED), asym_params_bytes(n, k, group_size)
    packed = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=src.device)
    params = torch.empty(max(nparams, 16), dtype=torch.uint8, device=src.device)
    sp = zp = 0
    if kind == SRC_I8_CODES:
        assert src.dtype == torch.uint8 and src_scales is not None and src_zeros is not None
        assert src_scales.dtype == torch.float32 and src_zeros.dtype == torch.uint8
        assert src_scales.is_contiguous() and src_zeros.is_contiguous()
        sp, zp = src_scales.data_ptr(), src_zeros.data_ptr()
    _check(lib().w4a8_pack_weights_asym(src.data_ptr(), kind, sp, zp, n, k, group_size, packed.data_ptr(),
                                        params.data_ptr(), _stream()), "w4a8_pack_weights_asym")
    return packed[:nbytes], params[:nparams]


def linear_asym(x8, x_scale, packed, params, n, group_size, out=None, out_dtype=torch.bfloat16):
    m, k = x8.shape
    assert x8.dtype == torch.uint8 and x8.stride(1) == 1
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x8.device)
    _check(lib().w4a8_linear_asym(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)), x_scale.data_ptr(),
                                  packed.data_ptr(), params.data_ptr(), n, group_size, out.data_ptr(), _dtype_code(out),
                                  out.stride(0) if m > 1 else max(n, out.stride(0)), _stream()), "w4a8_linear_asym")
    return out


def dequant_weights_asym(packed: torch.Tensor, params: torch.Tensor, n: int, k: int, group_size: int,
                         two_level: bool = False) -> torch.Tensor:
    w8 = torch.empty((n, k), dtype=torch.uint8, device=packed.device)
    fn = lib().w4a8_dequant_weights_asym_two_level if two_level else lib().w4a8_dequant_weights_asym
    _check(fn(packed.data_ptr(), params.data_ptr(), n, k, group_size, w8.data_ptr(), _stream()),
           "w4a8_dequant_weights_asym")
    return w8


def linear_asym_two_level(x8, x_scale, packed, params8, w_out_scales, n, group_size, out=None, out_dtype=torch.bfloat16):
    """w4a8_linear_asym_two_level; `w_out_scales` holds N floats (per channel) or one (per tensor)."""
    m, k = x8.shape
    if out is None:
        out = torch.empty((m, n), dtype=out_dtype, device=x8.device)
    per_channel = 1 if w_out_scales.numel() > 1 else 0
    assert w_out_scales.numel() in (1, n) and w_out_scales.dtype == torch.float32
    _check(lib().w4a8_linear_asym_two_level(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                            x_scale.data_ptr(), packed.data_ptr(), params8.data_ptr(),
                                            w_out_scales.data_ptr(), per_channel, n, group_size, out.data_ptr(),
                                            _dtype_code(out), out.stride(0) if m > 1 else max(n, out.stride(0)), _stream()),
           "w4a8_linear_asym_two_level")
    return out


def dequant_weights(packed: torch.Tensor, n: int, k: int, layout: int) -> torch.Tensor:
    w8 = torch.empty((n, k), dtype=torch.uint8, device=packed.device)
    _check(lib().w4a8_dequant_weights(packed.data_ptr(), n, k, layout, w8.data_ptr(), _stream()),
           "w4a8_dequant_weights")
    return w8


def silu_mul(gu: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    m, f2 = gu.shape
    f = f2 // 2
    assert gu.dtype == torch.bfloat16 and gu.stride(1) == 1 and f2 == 2 * f
    if out is None:
        out = torch.empty((m, f), dtype=torch.bfloat16, device=gu.device)
    _check(lib().w4a8_silu_mul(gu.data_ptr(), m, f, gu.stride(0) if m > 1 else max(f2, gu.stride(0)), out.data_ptr(),
                               out.stride(0) if m > 1 else max(f, out.stride(0)), _stream()), "w4a8_silu_mul")
    return out


def linear_fp8_out(x8, x_scale, packed, w_scales, n, group_size, y_scale, out=None):
    """w4a8_linear_fp8_out: the layer's bf16 output quantized with `y_scale` (the next layer's static scale)."""
    m, k = x8.shape
    assert x8.dtype == torch.uint8 and x8.stride(1) == 1 and y_scale.dtype == torch.float32
    if out is None:
        out = torch.empty((m, n), dtype=torch.uint8, device=x8.device)
    _check(lib().w4a8_linear_fp8_out(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                     x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), n, group_size,
                                     y_scale.data_ptr(), out.data_ptr(), out.stride(0) if m > 1 else max(n, out.stride(0)),
                                     _stream()), "w4a8_linear_fp8_out")
    return out


def interleave_gate_up(w_gate_up: torch.Tensor) -> torch.Tensor:
    """Row order w4a8_linear_silu_mul_fp8_out expects: [2F, K] with gate rows first, then up rows -> bands of 16 gate
    rows and the 16 up rows of the same channels in turn.  A pure re-ordering of rows (F % 16 == 0)."""
    f2, k = w_gate_up.shape
    f = f2 // 2
    assert f2 == 2 * f and f % 16 == 0
    return torch.stack([w_gate_up[:f].reshape(f // 16, 16, k), w_gate_up[f:].reshape(f // 16, 16, k)], dim=1).reshape(f2, k).contiguous()


def linear_silu_mul_fp8_out(x8, x_scale, packed, w_scales, f, group_size, h_scale, out=None):
    """w4a8_linear_silu_mul_fp8_out: packed/w_scales from the interleaved gate|up matrix; returns uint8 [M, F]."""
    m, k = x8.shape
    assert x8.dtype == torch.uint8 and x8.stride(1) == 1 and h_scale.dtype == torch.float32
    if out is None:
        out = torch.empty((m, f), dtype=torch.uint8, device=x8.device)
    _check(lib().w4a8_linear_silu_mul_fp8_out(x8.data_ptr(), m, k, x8.stride(0) if m > 1 else max(k, x8.stride(0)),
                                              x_scale.data_ptr(), packed.data_ptr(), w_scales.data_ptr(), f, group_size,
                                              h_scale.data_ptr(), out.data_ptr(),
                                              out.stride(0) if m > 1 else max(f, out.stride(0)), _stream()),
           "w4a8_linear_silu_mul_fp8_out")
    return out


def silu_mul_quantize(gu: torch.Tensor, scale: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    m, f2 = gu.shape
    f = f2 // 2
    assert gu.dtype == torch.bfloat16 and gu.stride(1) == 1 and f2 == 2 * f and scale.dtype == torch.float32
    if out is None:
        out = torch.empty((m, f), dtype=torch.uint8, device=gu.device)
    _check(lib().w4a8_silu_mul_quantize(gu.data_ptr(), m, f, gu.stride(0) if m > 1 else max(f2, gu.stride(0)),
                                        scale.data_ptr(), out.data_ptr(), out.stride(0) if m > 1 else max(f, out.stride(0)),
                                        _stream()), "w4a8_silu_mul_quantize")
    return out


def hessian_accumulate(x: torch.Tensor, h: torch.Tensor | None = None) -> torch.Tensor:
    """w4a8_hessian_accumulate: h (float32 [K, K], created as zeros when None) += x^T x for x [T, K] float32/bf16."""
    t, k = x.shape
    assert x.stride(1) == 1
    if h is None:
        h = torch.zeros((k, k), dtype=torch.float32, device=x.device)
    assert h.dtype == torch.float32 and h.is_contiguous() and tuple(h.shape) == (k, k)
    _check(lib().w4a8_hessian_accumulate(x.data_ptr(), _dtype_code(x), t, k, x.stride(0) if t > 1 else max(k, x.stride(0)),
                                         h.data_ptr(), _stream()), "w4a8_hessian_accumulate")
    return h


def hessian_inverse_factor(h: torch.Tensor, damp: float = 0.01, perm: torch.Tensor | None = None):
    """w4a8_hessian_inverse_factor: h float32 [K, K] -> (U float32 [K, K], info int32 [1]); info stays on the device
    (0 = success), so the call does not synchronize."""
    k = h.shape[0]
    assert h.dtype == torch.float32 and h.is_contiguous() and tuple(h.shape) == (k, k)
    assert perm is None or (perm.dtype == torch.int32 and perm.is_contiguous() and perm.numel() == k)
    nbytes = lib().w4a8_hessian_factor_workspace_bytes(k)
    if nbytes == 0:
        raise ValueError(f"w4a8_hessian_inverse_factor: unsupported K = {k}")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=h.device)
    u = torch.empty((k, k), dtype=torch.float32, device=h.device)
    info = torch.empty(1, dtype=torch.int32, device=h.device)
    _check(lib().w4a8_hessian_inverse_factor(h.data_ptr(), k, float(damp), perm.data_ptr() if perm is not None else None,
                                             ws.data_ptr(), nbytes, u.data_ptr(), info.data_ptr(), _stream()),
           "w4a8_hessian_inverse_factor")
    return u, info


def gar_permutation(h_diag: torch.Tensor, group_size: int) -> torch.Tensor:
    """w4a8_gar_permutation: h_diag float32 [K] on the device -> int32 [K]."""
    assert h_diag.dtype == torch.float32 and h_diag.is_contiguous()
    k = h_diag.numel()
    perm = torch.empty(k, dtype=torch.int32, device=h_diag.device)
    _check(lib().w4a8_gar_permutation(h_diag.data_ptr(), k, group_size, perm.data_ptr(), _stream()), "w4a8_gar_permutation")
    return perm


def dpq_calibrate(w: torch.Tensor, u_factor: torch.Tensor, w_scale: torch.Tensor, group_size: int,
                  perm: torch.Tensor | None = None, mse_grid: int = 0, mse_max_shrink: float = 0.8):
    """w4a8_dpq_calibrate (mse_grid <= 1) / w4a8_dpq_calibrate_mse.  w float32 [N, K]; u_factor float32 [K, K] (of the
    reordered columns when perm is given); w_scale float32 with N elements or one.  Returns (codes uint8 [N, K],
    scales8 float32 [N, K/G], zeros uint8 [N, K/G])."""
    n, k = w.shape
    assert w.dtype == torch.float32 and w.is_contiguous() and u_factor.dtype == torch.float32 and u_factor.is_contiguous()
    assert tuple(u_factor.shape) == (k, k) and w_scale.dtype == torch.float32 and w_scale.numel() in (1, n)
    assert perm is None or (perm.dtype == torch.int32 and perm.numel() == k)
    dev = w.device
    codes = torch.empty((n, k), dtype=torch.uint8, device=dev)
    scales = torch.empty((n, k // group_size), dtype=torch.float32, device=dev)
    zeros = torch.empty((n, k // group_size), dtype=torch.uint8, device=dev)
    nbytes = lib().w4a8_dpq_workspace_bytes(n, k)
    work = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=dev)
    per_channel = 1 if w_scale.numel() > 1 else 0
    perm_ptr = perm.data_ptr() if perm is not None else 0
    if mse_grid > 1:
        _check(lib().w4a8_dpq_calibrate_mse(w.data_ptr(), u_factor.data_ptr(), w_scale.data_ptr(), per_channel, perm_ptr, n, k,
                                            group_size, mse_grid, mse_max_shrink, codes.data_ptr(), scales.data_ptr(),
                                            zeros.data_ptr(), work.data_ptr(), nbytes, _stream()), "w4a8_dpq_calibrate_mse")
    else:
        _check(lib().w4a8_dpq_calibrate(w.data_ptr(), u_factor.data_ptr(), w_scale.data_ptr(), per_channel, perm_ptr, n, k,
                                        group_size, codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(), work.data_ptr(),
                                        nbytes, _stream()), "w4a8_dpq_calibrate")
    return codes, scales, zeros


def probe_stream_read(buf: torch.Tensor, sink: torch.Tensor) -> None:
    _check(lib().w4a8_probe_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream()),
           "w4a8_probe_stream_read")


def probe_mfma(iters: int, sink: torch.Tensor) -> float:
    """Enqueues the MFMA issue probe; returns the flop count of the call."""
    _check(lib().w4a8_probe_mfma_e4m3(iters, sink.data_ptr(), _stream()), "w4a8_probe_mfma_e4m3")
    return lib().w4a8_probe_mfma_flop(iters)
