"""Rank selection (Sec. 3.3): explained-variance ranks from the mode spectra of a stored activation,
the perplexity table of a set of layers, and the budgeted choice of one threshold per layer.

Every computation of the method runs in the HIP library behind the C ABI (asi_mode_spectrum,
asi_explained_variance_ranks, asi_core_project, asi_weight_grad_*, asi_frobenius_diff, asi_rank_select);
this file allocates the buffers and strings the calls together.  The exact weight gradient that a
perplexity is measured against is the caller's (the framework's own backward pass produces it).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as B

PAPER_THRESHOLDS = (0.4, 0.5, 0.6, 0.7, 0.8, 0.9)      # the set E of Sec. 4.1


def _dtype_name(t: torch.Tensor) -> str:
    if t.dtype == torch.float32:
        return "f32"
    if t.dtype == torch.bfloat16:
        return "bf16"
    raise TypeError("activations are fp32 or bf16")


@dataclass
class ModeSpectrum:
    eigenvalues: torch.Tensor      # fp64 (n), descending
    eigenvectors: torch.Tensor     # fp32 (n, n), column k = k-th principal component
    sweeps: int


def mode_spectrum(A: torch.Tensor, mode: int) -> ModeSpectrum:
    """Squared singular values and left singular vectors of the mode's unfolding (App. A.2)."""
    if not A.is_cuda:
        raise RuntimeError("the ASI path runs on the GPU only (no CPU fallback)")
    A = A.detach().contiguous()
    desc = B.make_desc(tuple(A.shape), (1,) * A.dim(), _dtype_name(A))
    need = B.asi_mode_spectrum_workspace_bytes(desc, mode)
    if need == 0:
        raise B.AsiError(2, "asi_mode_spectrum_workspace_bytes")
    n = A.shape[mode]
    ws = torch.empty(need, dtype=torch.uint8, device=A.device)
    lam = torch.empty(n, dtype=torch.float64, device=A.device)
    vec = torch.empty(n, n, dtype=torch.float32, device=A.device)
    sweeps = B.asi_mode_spectrum(desc, A, mode, lam, vec, ws)
    return ModeSpectrum(lam, vec, sweeps)


def explained_variance_ranks(spectra: Sequence[ModeSpectrum], eps: Sequence[float]) -> List[Tuple[int, ...]]:
    """One tuple of ranks (one per mode) per threshold: the layer's rows of the rank tensor R."""
    per_mode = []
    for sp in spectra:
        r = torch.empty(len(eps), dtype=torch.int32, device=sp.eigenvalues.device)
        B.asi_explained_variance_ranks(sp.eigenvalues, eps, r)
        per_mode.append(r)
    host = [r.cpu().tolist() for r in per_mode]
    return [tuple(int(h[j]) for h in host) for j in range(len(eps))]


def hosvd_factors(spectra: Sequence[ModeSpectrum], ranks: Sequence[int]) -> List[torch.Tensor]:
    """Factors of the truncated HOSVD: the leading ranks[m] principal components of every mode."""
    return [sp.eigenvectors[:, :r].contiguous() for sp, r in zip(spectra, ranks)]


@dataclass
class LayerTable:
    ranks: List[Tuple[int, ...]]   # per threshold
    memory: List[int]              # Eq. 5 per threshold, in elements
    perplexity: List[float]        # Eq. 7 per threshold


def perplexity_row(A: torch.Tensor, grad_out: torch.Tensor, dW_exact: torch.Tensor, eps: Sequence[float] = PAPER_THRESHOLDS,
                   conv: Optional[B.Conv2dDesc] = None, dout: int = 0) -> LayerTable:
    """One layer's row of the perplexity matrix P and of the rank tensor R (Sec. 3.3, Steps 1 and 2):
    per threshold, truncate the HOSVD of A, compute the weight gradient from the compressed form and
    take its Frobenius distance to the exact one."""
    A = A.detach().contiguous()
    grad_out = grad_out.detach().contiguous().to(A.dtype)
    dW_exact = dW_exact.detach().contiguous().float()
    spectra = [mode_spectrum(A, m) for m in range(A.dim())]
    rank_rows = explained_variance_ranks(spectra, eps)
    f32 = dict(dtype=torch.float32, device=A.device)
    fws = torch.empty(B.FROBENIUS_WS_BYTES, dtype=torch.uint8, device=A.device)
    out = torch.empty(1, dtype=torch.float64, device=A.device)
    table = LayerTable([], [], [])
    done = {}
    for ranks in rank_rows:
        if ranks not in done:
            desc = B.make_desc(tuple(A.shape), ranks, _dtype_name(A))
            ws = B.alloc_workspace(desc, conv, dout, device=A.device)
            U = hosvd_factors(spectra, ranks)
            S = torch.empty(ranks, **f32)
            B.asi_core_project(desc, A, U, S, ws)
            dW = torch.empty(dW_exact.shape, **f32)
            if conv is not None:
                B.asi_weight_grad_conv2d(desc, S, U, grad_out, conv, dW, False, ws)
            else:
                B.asi_weight_grad_linear(desc, S, U, grad_out, dout, dW, False, ws)
            B.asi_frobenius_diff(dW_exact, dW, out, fws)
            done[ranks] = (B.asi_activation_memory(desc), float(out.item()))
        mem, ppl = done[ranks]
        table.ranks.append(ranks)
        table.memory.append(mem)
        table.perplexity.append(ppl)
    return table


def select_ranks(tables: Sequence[LayerTable], budget: int) -> Tuple[List[Tuple[int, ...]], List[int], float]:
    """Eq. 8-9: the ranks of every layer under a budget of `budget` elements.  Returns (ranks per layer,
    threshold index per layer, total perplexity); raises AsiError(ASI_ERR_INFEASIBLE) if nothing fits."""
    choice, total = B.asi_rank_select([t.perplexity for t in tables], [t.memory for t in tables], budget)
    return [t.ranks[j] for t, j in zip(tables, choice)], choice, total
