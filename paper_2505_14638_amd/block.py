"""The decoder-block linear stack (QKV -> O -> gate|up -> SiLU*mul -> down) on the HIP path.

Orchestration only: every tensor operation is one call into the C-ABI library (activation quantization, linear
layer, SiLU*mul); PyTorch provides buffers and views.  The O projection reads the first `hidden` columns of the QKV
output (a strided view -- the quantizer takes a row stride), standing in for attention, which is not part of the
quantized-linear path.  Intermediates are bf16, each linear layer's input is quantized to FP8 with its own static
per-tensor scale (Eq. 13; all linear layers of a block are quantized, Sec. 4.1).

`fused=True` runs the same computation with the quantization of each intermediate folded into the kernel that produces
it (w4a8_linear_fp8_out for QKV and O, w4a8_linear_silu_mul_fp8_out for gate|up with SiLU*mul, on a row-interleaved
copy of the gate|up weights) and, up to eight tokens, the quantization of the block input folded into the QKV layer
(w4a8_linear_quantize_in_fp8_out): four or five launches instead of nine, the same bytes at every layer input and the
same block output.
"""
from __future__ import annotations

import torch

from . import binding as B

LAYERS = ("qkv", "o", "gate_up", "down")


class DecoderBlockLinears:
    def __init__(self, hidden: int, ffn: int, qkv_out: int, group_size: int = 128, device: str = "cuda:0",
                 fused: bool = False):
        self.hidden, self.ffn, self.group_size, self.device, self.fused = hidden, ffn, group_size, device, fused
        self.dims = {"qkv": (hidden, qkv_out), "o": (hidden, hidden), "gate_up": (hidden, 2 * ffn), "down": (ffn, hidden)}
        self.weights = {}
        self.scales_x = {}
        self._buffers = {}
        self.quantize_in_up_to = 8                               # tokens up to which the QKV layer quantizes its own input
        self._workspace = None                                   # scratch of w4a8_linear (K ranges across workgroups), grown on demand
        self._retired = []                                       # outgrown workspaces, kept for launches already captured

    def load_layer(self, name: str, w_f32: torch.Tensor) -> None:
        """Quantize (round-to-nearest INT4) and pack one [N, K] float32 weight matrix on the device."""
        k, n = self.dims[name]
        assert tuple(w_f32.shape) == (n, k)
        w_dev = w_f32.to(self.device)
        self.weights[name] = B.pack_weights(w_dev, self.group_size, B.LAYOUT_TILED)
        if name == "gate_up":                                    # row-interleaved copy for the fused gate|up + SiLU*mul layer
            self.weights["gate_up_interleaved"] = B.pack_weights(B.interleave_gate_up(w_dev), self.group_size, B.LAYOUT_TILED)

    def set_act_scale(self, name: str, s_x: float) -> None:
        self.scales_x[name] = torch.tensor([s_x], dtype=torch.float32, device=self.device)

    def _buf(self, key, shape, dtype):
        b = self._buffers.get(key)
        if b is None or tuple(b.shape) != tuple(shape):
            b = torch.empty(shape, dtype=dtype, device=self.device)
            self._buffers[key] = b
        return b

    def _ws(self, name: str, m: int):
        """The workspace w4a8_linear asks for on this layer at this batch size (None where it asks for none)."""
        k, n = self.dims[name]
        need = B.linear_workspace_bytes(m, k, n, self.group_size)
        if need == 0:
            return None
        if self._workspace is None or self._workspace.numel() < need:
            if self._workspace is not None:
                self._retired.append(self._workspace)            # a captured graph may still write to it: never freed
            self._workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._workspace

    def _linear(self, name: str, x: torch.Tensor, m: int) -> torch.Tensor:
        k, n = self.dims[name]
        x8 = self._buf((name, "x8", m), (m, k), torch.uint8)
        y = self._buf((name, "y", m), (m, n), torch.bfloat16)
        B.quantize_act(x, self.scales_x[name], out=x8)
        packed, scales = self.weights[name]
        # only the last layer takes the workspace: the fused forms of the others take none, and with one w4a8_linear may add
        # the ranges of K in another order than they do
        ws = self._ws(name, m) if name == "down" else None
        B.linear(x8, self.scales_x[name], packed, scales, n, self.group_size, B.LAYOUT_TILED, out=y, workspace=ws)
        return y

    def _forward_fused(self, x: torch.Tensor, keep: dict | None) -> torch.Tensor:
        m, g, sx, w = x.shape[0], self.group_size, self.scales_x, self.weights
        x8 = self._buf(("qkv", "x8", m), (m, self.hidden), torch.uint8)
        qkv8 = self._buf(("qkv", "y8", m), (m, self.dims["qkv"][1]), torch.uint8)
        if m <= self.quantize_in_up_to and m * self.hidden <= 65536:   # every workgroup quantizes x itself: one launch fewer
            B.linear_quantize_in_fp8_out(x, sx["qkv"], *w["qkv"], self.dims["qkv"][1], g, sx["o"], out=qkv8,
                                         x8_out=x8 if keep is not None else None)
        else:
            B.quantize_act(x, sx["qkv"], out=x8)
            B.linear_fp8_out(x8, sx["qkv"], *w["qkv"], self.dims["qkv"][1], g, sx["o"], out=qkv8)
        o8 = B.linear_fp8_out(qkv8[:, :self.hidden], sx["o"], *w["o"], self.hidden, g, sx["gate_up"],
                              out=self._buf(("o", "y8", m), (m, self.hidden), torch.uint8))
        h8 = self._buf(("h8", m), (m, self.ffn), torch.uint8)
        B.linear_silu_mul_fp8_out(o8, sx["gate_up"], *w["gate_up_interleaved"], self.ffn, g, sx["down"], out=h8)
        y = B.linear(h8, sx["down"], *w["down"], self.hidden, g, B.LAYOUT_TILED,
                     out=self._buf(("down", "y", m), (m, self.hidden), torch.bfloat16), workspace=self._ws("down", m))
        if keep is not None:
            keep.update(qkv_x8=x8, o_x8=qkv8[:, :self.hidden], gate_up_x8=o8, down_x8=h8, down=y)
        return y

    def forward(self, x: torch.Tensor, keep: dict | None = None) -> torch.Tensor:
        """x: bf16 [M, hidden] on the device.  `keep`, if given, receives every intermediate tensor."""
        if self.fused:
            return self._forward_fused(x, keep)
        m = x.shape[0]
        qkv = self._linear("qkv", x, m)
        o = self._linear("o", qkv[:, :self.hidden], m)
        gu = self._linear("gate_up", o, m)
        h = B.silu_mul(gu, out=self._buf(("h", m), (m, self.ffn), torch.bfloat16))
        y = self._linear("down", h, m)
        if keep is not None:
            keep.update(qkv=qkv, o=o, gate_up=gu, h=h, down=y,
                        **{nm + "_x8": self._buffers[(nm, "x8", m)] for nm in LAYERS})
        return y
