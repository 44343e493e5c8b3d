"""Training-loop integration: conv2d / linear layers whose backward pass keeps the compressed
activation (core S and factors U, Eq. 3) instead of the activation A itself (Sec. 3.2, Alg. 1).

Forward:  y = conv2d(x, W) (or x W^T) by the framework's own operator, which is not part of the
          method; then U <- asi_compress (warm-started from the layer's previous factors; the very
          first call takes Alg. 1's t = 0 branch, asi_compress_cold) and S <- asi_core_project.  Only
          (S, U) are saved for backward.
Backward: dW from (S, U, dy) by asi_weight_grad_conv2d / asi_weight_grad_linear (Eq. 14); dx needs only
          W and dy (Eq. 2) and stays the framework's operator; db = sum of dy.

All arithmetic of the method runs in the HIP library behind the C ABI; this file only keeps the
per-layer state (previous factors, workspace) and wires the calls into autograd.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch
import torch.nn.functional as F

from . import binding as B


# One workspace per device, grown to the largest layer: the calls of all layers are ordered on the
# stream, and nothing in the workspace outlives a call.
_WORKSPACE = {}


def _workspace(device: torch.device, nbytes: int) -> torch.Tensor:
    ws = _WORKSPACE.get(device)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _WORKSPACE[device] = ws
    return ws


class AsiState:
    """Per-layer state of Alg. 1: the factors of the previous training step and the workspace."""

    def __init__(self, ranks: Sequence[int], seed: int = 0):
        self.ranks = tuple(int(r) for r in ranks)
        self.seed = int(seed)
        self.U_prev: Optional[List[torch.Tensor]] = None
        self.shape = None
        self.desc = None
        self.ws_bytes = 0
        self.info = None

    def _prepare(self, x: torch.Tensor, conv: Optional[B.Conv2dDesc], dout: int):
        key = (tuple(x.shape), x.dtype)
        if key == self.shape:
            return
        if x.dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("ASI layers take fp32 or bf16 activations")
        if len(self.ranks) != x.dim():
            raise ValueError(f"{len(self.ranks)} ranks for a {x.dim()}-mode activation")
        self.shape = key
        self.desc = B.make_desc(tuple(x.shape), self.ranks, "f32" if x.dtype == torch.float32 else "bf16")
        self.ws_bytes = B.asi_workspace_bytes(self.desc, conv, dout)
        if self.ws_bytes == 0:
            raise B.AsiError(1, "asi_workspace_bytes")
        self.info = torch.zeros(1, dtype=torch.int32, device=x.device)
        self.U_prev = None                      # another shape: start again from the cold branch

    def compress(self, x: torch.Tensor, conv: Optional[B.Conv2dDesc], dout: int):
        """One step of Alg. 1 on x.  Returns (S, U); U also becomes the next step's warm start."""
        if not x.is_cuda:
            raise RuntimeError("the ASI path runs on the GPU only (no CPU fallback)")
        x = x.detach().contiguous()
        self._prepare(x, conv, dout)
        f32 = dict(dtype=torch.float32, device=x.device)
        ws = _workspace(x.device, self.ws_bytes)
        U = [torch.empty(n, r, **f32) for n, r in zip(x.shape, self.ranks)]
        if self.U_prev is None:
            B.asi_compress_cold(self.desc, x, self.seed, U, ws, self.info)
        else:
            B.asi_compress(self.desc, x, self.U_prev, U, ws, self.info)
        S = torch.empty(self.ranks, **f32)
        B.asi_core_project(self.desc, x, U, S, ws)
        self.U_prev = U
        return S, U


class _AsiConv2dFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, state: AsiState, stride, padding, dilation, groups):
        y = F.conv2d(x, weight, bias, stride, padding, dilation, groups)
        conv = B.make_conv(weight.shape[0], weight.shape[2], weight.shape[3], stride, padding, dilation, groups)
        S, U = state.compress(x, conv, 0)
        ctx.save_for_backward(weight, S, *U)            # not x: that is the point
        ctx.desc, ctx.ws_bytes, ctx.act_dtype, ctx.conv = state.desc, state.ws_bytes, x.dtype, conv
        ctx.x_shape, ctx.has_bias = tuple(x.shape), bias is not None      # dy is passed in the activation's dtype
        ctx.geom = (stride, padding, dilation, groups)
        return y

    @staticmethod
    def backward(ctx, gy):
        weight, S, *U = ctx.saved_tensors
        stride, padding, dilation, groups = ctx.geom
        gy = gy.contiguous()
        gx = gw = gb = None
        if ctx.needs_input_grad[0]:
            gx = torch.nn.grad.conv2d_input(ctx.x_shape, weight, gy, stride, padding, dilation, groups)
        if ctx.needs_input_grad[1]:
            dW = torch.empty(weight.shape, dtype=torch.float32, device=gy.device)
            B.asi_weight_grad_conv2d(ctx.desc, S, U, gy.to(ctx.act_dtype), ctx.conv, dW, False,
                                     _workspace(gy.device, ctx.ws_bytes))
            gw = dW.to(weight.dtype)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            gb = gy.sum((0, 2, 3))
        return gx, gw, gb, None, None, None, None, None


class _AsiLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, state: AsiState):
        y = F.linear(x, weight, bias)
        S, U = state.compress(x, None, weight.shape[0])
        ctx.save_for_backward(weight, S, *U)
        ctx.desc, ctx.ws_bytes, ctx.act_dtype, ctx.has_bias = state.desc, state.ws_bytes, x.dtype, bias is not None
        return y

    @staticmethod
    def backward(ctx, gy):
        weight, S, *U = ctx.saved_tensors
        gy = gy.contiguous()
        gx = gw = gb = None
        if ctx.needs_input_grad[0]:
            gx = gy.matmul(weight)
        if ctx.needs_input_grad[1]:
            dW = torch.empty(weight.shape, dtype=torch.float32, device=gy.device)
            B.asi_weight_grad_linear(ctx.desc, S, U, gy.to(ctx.act_dtype), weight.shape[0], dW, False,
                                     _workspace(gy.device, ctx.ws_bytes))
            gw = dW.to(weight.dtype)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            gb = gy.sum((0, 1))
        return gx, gw, gb, None


class AsiConv2d(torch.nn.Conv2d):
    """nn.Conv2d whose weight gradient comes from the compressed activation.  `ranks` = (r_B, r_C, r_H, r_W)."""

    def __init__(self, *args, ranks: Sequence[int], seed: int = 0, **kw):
        super().__init__(*args, **kw)
        if self.padding_mode != "zeros" or isinstance(self.padding, str):
            raise ValueError("AsiConv2d supports explicit zero padding")
        self.asi = AsiState(ranks, seed)

    def forward(self, x):
        if not (self.training and torch.is_grad_enabled() and self.weight.requires_grad):
            return super().forward(x)
        return _AsiConv2dFn.apply(x, self.weight, self.bias, self.asi, tuple(self.stride), tuple(self.padding),
                                  tuple(self.dilation), self.groups)


class AsiLinear(torch.nn.Linear):
    """nn.Linear on (B, N, D) activations whose weight gradient comes from the compressed activation."""

    def __init__(self, *args, ranks: Sequence[int], seed: int = 0, **kw):
        super().__init__(*args, **kw)
        self.asi = AsiState(ranks, seed)

    def forward(self, x):
        if not (self.training and torch.is_grad_enabled() and self.weight.requires_grad):
            return super().forward(x)
        if x.dim() != 3:
            raise ValueError("AsiLinear takes (batch, tokens, features) activations")
        return _AsiLinearFn.apply(x, self.weight, self.bias, self.asi)
