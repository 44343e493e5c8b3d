"""Per-layer driver around the C ABI: owns the device buffers of one layer
(factors, core, weight gradient, workspace) and issues the calls of one
training step.  No arithmetic happens here.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def to_device(values_f32: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Upload an array whose values are already exactly representable in `dtype`."""
    t = torch.from_numpy(np.ascontiguousarray(values_f32, dtype=np.float32)).to(device)
    if dtype == "bf16":
        t = t.to(torch.bfloat16)      # exact: the values were rounded to bf16 on the host
    return t.contiguous()


class LayerRunner:
    """Device state and calls for one fine-tuned layer.

    `layer` needs the attributes dims, ranks, dtype ("f32"/"bf16"), kind
    ("conv2d"/"linear"), cout, k, stride, pad, dil, groups, dw_shape.
    """

    def __init__(self, layer, device="cuda"):
        self.layer = layer
        self.device = device
        self.desc = B.make_desc(layer.dims, layer.ranks, layer.dtype)
        self.conv = None
        self.dout = 0
        if layer.kind == "conv2d":
            self.conv = B.make_conv(layer.cout, layer.k, layer.k, (layer.stride,) * 2, (layer.pad,) * 2,
                                    (layer.dil,) * 2, layer.groups)
        else:
            self.dout = layer.cout
        self.ws = B.alloc_workspace(self.desc, self.conv, self.dout, device)
        f32 = dict(dtype=torch.float32, device=device)
        self.U = [[torch.zeros(n, r, **f32) for n, r in zip(layer.dims, layer.ranks)] for _ in range(2)]
        self.cur = 0                       # which of the two factor sets holds the latest basis
        self.S = torch.zeros(tuple(layer.ranks), **f32)
        self.dW = torch.zeros(tuple(layer.dw_shape), **f32)
        self.info = torch.zeros(1, dtype=torch.int32, device=device)

    # -- state ---------------------------------------------------------------
    def set_factors(self, U: Sequence[np.ndarray]) -> None:
        for dst, src in zip(self.U[self.cur], U):
            dst.copy_(torch.from_numpy(np.ascontiguousarray(src, dtype=np.float32)))

    def factors(self) -> List[torch.Tensor]:
        return self.U[self.cur]

    def upload(self, values_f32: np.ndarray) -> torch.Tensor:
        return to_device(values_f32, self.layer.dtype, self.device)

    # -- the calls of one step -------------------------------------------------
    def compress(self, A: torch.Tensor) -> List[torch.Tensor]:
        """U <- one warm-started subspace step from the current factors."""
        prev, out = self.U[self.cur], self.U[1 - self.cur]
        B.asi_compress(self.desc, A, prev, out, self.ws, self.info)
        self.cur = 1 - self.cur
        return out

    def compress_cold(self, A: torch.Tensor, seed: int) -> List[torch.Tensor]:
        """U <- the first iteration of Alg. 1: the subspace step from a generated standard-normal V."""
        out = self.U[1 - self.cur]
        B.asi_compress_cold(self.desc, A, seed, out, self.ws, self.info)
        self.cur = 1 - self.cur
        return out

    def core(self, A: torch.Tensor, U: Optional[Sequence[torch.Tensor]] = None) -> torch.Tensor:
        B.asi_core_project(self.desc, A, U if U is not None else self.U[self.cur], self.S, self.ws)
        return self.S

    def weight_grad(self, grad_out: torch.Tensor, S: Optional[torch.Tensor] = None,
                    U: Optional[Sequence[torch.Tensor]] = None, accumulate: bool = False) -> torch.Tensor:
        S = self.S if S is None else S
        U = self.U[self.cur] if U is None else U
        if self.conv is not None:
            B.asi_weight_grad_conv2d(self.desc, S, U, grad_out, self.conv, self.dW, accumulate, self.ws)
        else:
            B.asi_weight_grad_linear(self.desc, S, U, grad_out, self.dout, self.dW, accumulate, self.ws)
        return self.dW

    def step(self, A: torch.Tensor, grad_out: torch.Tensor) -> torch.Tensor:
        """The whole hot path for one layer and one training step."""
        self.compress(A)
        self.core(A)
        return self.weight_grad(grad_out)


class BatchRunner:
    """Several layers stepped together through the batched entry points: every kernel launch
    serves all of them.  Owns one LayerRunner per layer for the device buffers."""

    def __init__(self, layers, device="cuda"):
        if not 1 <= len(layers) <= B.MAX_BATCH:
            raise ValueError(f"1..{B.MAX_BATCH} layers per batch")
        self.runs = [LayerRunner(lay, device) for lay in layers]
        kinds = {r.layer.kind for r in self.runs}
        if len(kinds) != 1:
            raise ValueError("a batch holds conv2d layers or linear layers, not both")
        self.kind = kinds.pop()

    def compress(self, A: Sequence[torch.Tensor]) -> None:
        rs = self.runs
        B.asi_compress_batch([r.desc for r in rs], A, [r.U[r.cur] for r in rs], [r.U[1 - r.cur] for r in rs],
                             [r.ws for r in rs], [r.info for r in rs])
        for r in rs:
            r.cur = 1 - r.cur

    def core(self, A: Sequence[torch.Tensor]) -> None:
        rs = self.runs
        B.asi_core_project_batch([r.desc for r in rs], A, [r.U[r.cur] for r in rs], [r.S for r in rs],
                                 [r.ws for r in rs])

    def weight_grad(self, grad_out: Sequence[torch.Tensor], accumulate: bool = False) -> List[torch.Tensor]:
        rs = self.runs
        acc = [accumulate] * len(rs)
        if self.kind == "conv2d":
            B.asi_weight_grad_conv2d_batch([r.desc for r in rs], [r.S for r in rs], [r.U[r.cur] for r in rs], grad_out,
                                           [r.conv for r in rs], [r.dW for r in rs], acc, [r.ws for r in rs])
        else:
            B.asi_weight_grad_linear_batch([r.desc for r in rs], [r.S for r in rs], [r.U[r.cur] for r in rs], grad_out,
                                           [r.dout for r in rs], [r.dW for r in rs], acc, [r.ws for r in rs])
        return [r.dW for r in rs]

    def step(self, A: Sequence[torch.Tensor], grad_out: Sequence[torch.Tensor]) -> List[torch.Tensor]:
        self.compress(A)
        self.core(A)
        return self.weight_grad(grad_out)
