"""Seeded generators for activations, output gradients and warm-start bases.

Recipe (all draws from numpy's PCG64, float64, then rounded to the storage
dtype; whoever consumes the tensors reads the *rounded* values):
  1. true factors: Q of the QR of an (n_m x r_m) standard-normal matrix;
  2. core g[i_1..i_d] * prod_m (i_m+1)^(-alpha), g ~ N(0,1)  (alpha = 0: plain Gaussian);
  3. clean tensor = core expanded by the factors, scaled to unit RMS, plus
     noise_std * N(0,1);
  4. drift: before step t >= 1 every true factor is rotated by a Cayley
     rotation exp-like map of theta * K_t, K_t a fresh antisymmetric matrix of
     spectral norm 1; the core stays fixed, the noise is redrawn;
  5. warm-start basis for step 0: seeded random orthonormal (n_m x r_m);
  6. grad_out ~ N(0,1) in the layer's output shape.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from .configs import Layer

SEED_BASE = 50860000


def make_seed(cfg: int, layer: int, step: int) -> int:
    return SEED_BASE + 10000 * cfg + 100 * layer + step


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float64 array to the storage dtype and return the rounded values as float32."""
    x32 = x64.astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x32))
    raise ValueError(dtype)


def random_orthonormal(rng: np.random.Generator, n: int, r: int) -> np.ndarray:
    q, rr = np.linalg.qr(rng.standard_normal((n, r)))
    return q * np.sign(np.diag(rr))


def _expand(core: np.ndarray, factors: Sequence[np.ndarray]) -> np.ndarray:
    x = core
    for m, f in enumerate(factors):
        x = np.moveaxis(np.tensordot(f, x, axes=([1], [m])), 0, m)
    return x


def tucker_tensor(rng: np.random.Generator, dims, ranks, alpha: float,
                  factors: Sequence[np.ndarray] = None) -> Tuple[np.ndarray, List[np.ndarray], np.ndarray]:
    """Clean Tucker tensor of unit RMS.  Returns (tensor, factors, scaled core)."""
    if factors is None:
        factors = [random_orthonormal(rng, n, r) for n, r in zip(dims, ranks)]
    core = rng.standard_normal(tuple(ranks))
    for m, r in enumerate(ranks):
        w = np.arange(1, r + 1, dtype=np.float64) ** (-alpha)
        core = core * w.reshape([-1 if k == m else 1 for k in range(len(ranks))])
    x = _expand(core, factors)
    s = 1.0 / np.sqrt(np.mean(x * x))
    return x * s, list(factors), core * s


def cayley_rotation(rng: np.random.Generator, n: int, theta: float) -> np.ndarray:
    """Exactly orthogonal (I - tK/2)^-1 (I + tK/2), K antisymmetric with spectral norm 1."""
    m = rng.standard_normal((n, n))
    k = m - m.T
    nrm = np.linalg.norm(k, 2)
    if nrm > 0:
        k = k / nrm
    i = np.eye(n)
    return np.linalg.solve(i - 0.5 * theta * k, i + 0.5 * theta * k)


class LayerStream:
    """The sequence of (activation, grad_out) a layer sees over training steps."""

    def __init__(self, cfg: int, layer_index: int, layer: Layer, theta: float = 0.02):
        self.cfg, self.layer_index, self.layer, self.theta = cfg, layer_index, layer, theta
        ss = np.random.SeedSequence(make_seed(cfg, layer_index, 0))
        s_fac, s_core, s_u0 = ss.spawn(3)
        rng = np.random.default_rng(s_fac)
        self.factors0 = [random_orthonormal(rng, n, r) for n, r in zip(layer.dims, layer.ranks)]
        rngc = np.random.default_rng(s_core)
        core = rngc.standard_normal(tuple(layer.ranks))
        for m, r in enumerate(layer.ranks):
            w = np.arange(1, r + 1, dtype=np.float64) ** (-layer.alpha)
            core = core * w.reshape([-1 if k == m else 1 for k in range(len(layer.ranks))])
        self.core = core
        self._s_u0 = s_u0
        self._step = 0
        self._factors = [f.copy() for f in self.factors0]

    # -- true factors at a step (rotations applied cumulatively) ------------
    def _advance_to(self, step: int) -> None:
        if step < self._step:
            self._step = 0
            self._factors = [f.copy() for f in self.factors0]
        while self._step < step:
            self._step += 1
            ss = np.random.SeedSequence(make_seed(self.cfg, self.layer_index, self._step))
            rng = np.random.default_rng(ss.spawn(3)[2])
            for m, f in enumerate(self._factors):
                self._factors[m] = cayley_rotation(rng, f.shape[0], self.theta) @ f

    def true_factors(self, step: int) -> List[np.ndarray]:
        self._advance_to(step)
        return [f.copy() for f in self._factors]

    def activation(self, step: int = 0) -> np.ndarray:
        """Activation at `step`, rounded to the layer's dtype, values returned as float32."""
        self._advance_to(step)
        ss = np.random.SeedSequence(make_seed(self.cfg, self.layer_index, step))
        rng = np.random.default_rng(ss.spawn(3)[0])
        x = _expand(self.core, self._factors)
        x *= 1.0 / np.sqrt(np.mean(x * x))
        if self.layer.noise > 0:
            x += self.layer.noise * rng.standard_normal(x.shape)
        return round_to_dtype(x, self.layer.dtype)

    def grad_out(self, step: int = 0) -> np.ndarray:
        ss = np.random.SeedSequence(make_seed(self.cfg, self.layer_index, step))
        rng = np.random.default_rng(ss.spawn(3)[1])
        return round_to_dtype(rng.standard_normal(self.layer.grad_out_shape), self.layer.dtype)

    def u_prev0(self) -> List[np.ndarray]:
        """Warm-start bases handed to step 0 (float32, orthonormal up to float32 rounding)."""
        rng = np.random.default_rng(self._s_u0)
        return [random_orthonormal(rng, n, r).astype(np.float32)
                for n, r in zip(self.layer.dims, self.layer.ranks)]
