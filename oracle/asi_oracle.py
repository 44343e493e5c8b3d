"""Float64 CPU oracle for the hot path of Activation Subspace Iteration (ASI).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, float64 NumPy statement of
what the method computes, written from the paper (arxiv 2505.05086).  Only the
tests, the smoke check and the CPU-baseline leg of the benchmark may call it;
the GPU library never does, and the two share no code.

Every function cites the passage of the paper it follows.  Where the method
reaches a result that has a plain definition (core projection, weight
gradients) the oracle is that definition written out; the subspace step is an
iteration, so it takes the algorithm's steps in the paper's order.

Readings of ambiguous passages (each is also listed in the design notes):
  * Alg. 1 computes V from "U^(t)" before assigning U^(t): that factor is the
    one kept from the previous step, U^(t-1).
  * Alg. 1's "S = S x_m U" must shrink mode m, so with Eq. 4's convention
    (matrix of shape Q x P_m maps mode size P_m to Q) the matrix is U^T.
  * Eq. 4's summand carries the output index where the summed one belongs; the
    standard m-mode product is meant.
  * Every mode is unfolded from the original activation (Alg. 1 says so), not
    from the partially projected core, so the modes are independent.
  * "Orthogonalize" is Gram-Schmidt (App. A.1); the sign/rotation freedom is
    fixed by taking the Q factor of the thin QR with positive diagonal R.
  * At t = 0 Alg. 1 draws V from a standard normal distribution; the draw is a
    counter-based generator (Philox4x32-10 + Box-Muller, see gaussian_V) so that
    both sides of a parity test produce the same V without storing it.
  * The backward formulation is given only as the cost sum C_ASI (Eq. 14); the
    contraction order is read off its five terms.
  * "FLOPs" in the paper are multiply-accumulates.

Parity pins: every function here is pinned by tests/test_oracle_pins.py (none
is "parity unpinned").
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


class OrthogonalizeBreakdown(ArithmeticError):
    """Raised when P has (numerically) dependent columns: no basis is invented."""

    def __init__(self, column: int):
        super().__init__(f"orthogonalisation broke down at column {column}")
        self.column = column


# --------------------------------------------------------------------------
# Sec. 3.2: unfolding and the m-mode product
# --------------------------------------------------------------------------
def unfold(A: np.ndarray, m: int) -> np.ndarray:
    """Mode-m unfolding A_m of shape (a_m, b_m) (Sec. 3.2, first paragraph).

    Row index = index along mode m (0-based here); the column index enumerates
    all remaining indices in row-major order.  Nothing downstream depends on
    that column order.
    """
    A = np.asarray(A, dtype=F64)
    return np.moveaxis(A, m, 0).reshape(A.shape[m], -1)


def mode_product(G: np.ndarray, Bmat: np.ndarray, m: int) -> np.ndarray:
    """m-mode product G x_m B with B of shape (Q, P_m) (Eq. 4).

    R[p_1..q..p_n] = sum_{p_m} G[p_1..p_m..p_n] * B[q, p_m].
    """
    G = np.asarray(G, dtype=F64)
    Bmat = np.asarray(Bmat, dtype=F64)
    if Bmat.ndim != 2 or Bmat.shape[1] != G.shape[m]:
        raise ValueError("mode_product: B must be (Q, P_m)")
    R = np.tensordot(Bmat, G, axes=([1], [m]))  # result has q first
    return np.moveaxis(R, 0, m)


# --------------------------------------------------------------------------
# Alg. 1 / App. A.1: one warm-started subspace-iteration step per mode
# --------------------------------------------------------------------------
def orthogonalize(P: np.ndarray, breakdown_rel: float = 1e-12) -> np.ndarray:
    """Orthonormal basis of range(P) by Gram-Schmidt (Alg. 1; App. A.1).

    Modified Gram-Schmidt applied twice.  Column j is made orthogonal to the
    finished columns 0..j-1 and normalised, which is exactly the Q factor of
    the thin QR of P with positive diagonal R.  A column whose remaining norm
    falls below breakdown_rel * ||P||_F raises OrthogonalizeBreakdown.
    """
    P = np.array(P, dtype=F64, copy=True)
    n, r = P.shape
    if r > n:
        raise ValueError("orthogonalize: more columns than rows")
    scale = math.sqrt(float(np.sum(P * P)))
    Q = np.zeros((n, r), dtype=F64)
    for j in range(r):
        v = P[:, j].copy()
        for _sweep in range(2):
            for k in range(j):
                v -= np.dot(Q[:, k], v) * Q[:, k]
        nv = math.sqrt(float(np.dot(v, v)))
        if not np.isfinite(nv) or nv <= breakdown_rel * scale:
            raise OrthogonalizeBreakdown(j)
        Q[:, j] = v / nv
    return Q


def subspace_step(A: np.ndarray, U_prev: np.ndarray, m: int) -> np.ndarray:
    """One warm-started subspace-iteration step on the mode-m unfolding (Alg. 1).

    V = A_m^T U_prev;  P = A_m V;  U = Orthogonalize(P).
    U_prev is the factor stored at the previous training step.
    """
    Am = unfold(A, m)
    U_prev = np.asarray(U_prev, dtype=F64)
    if U_prev.shape[0] != Am.shape[0]:
        raise ValueError("subspace_step: U_prev must be (a_m, r_m)")
    V = Am.T @ U_prev          # (b_m, r_m)
    P = Am @ V                 # (a_m, r_m)
    return orthogonalize(P)


def subspace_P(A: np.ndarray, U_prev: np.ndarray, m: int) -> np.ndarray:
    """The un-orthogonalised iterate P = A_m (A_m^T U_prev) of Alg. 1 (for tests)."""
    Am = unfold(A, m)
    return Am @ (Am.T @ np.asarray(U_prev, dtype=F64))


# --------------------------------------------------------------------------
# Alg. 1, branch t = 0: V is drawn i.i.d. standard normal instead of A_m^T U_prev
# --------------------------------------------------------------------------
# The draw must be reproducible on both sides of a parity test without storing V (b_m x r_m values), so
# it is a counter-based generator: Philox4x32-10 (Salmon et al., "Parallel random numbers: as easy as
# 1, 2, 3", SC 2011) keyed by the 64-bit seed, one call per (unfolding column c, group of four rank
# columns g, mode m) with counter (c mod 2^32, c div 2^32, g, m).  Its four 32-bit words give two pairs of
# uniforms u = (top 23 bits + 0.5) / 2^23 and each pair one Box-Muller pair
#     z0 = sqrt(-2 ln u1) cos(2 pi u2),  z1 = sqrt(-2 ln u1) sin(2 pi u2),
# so V[c, 4 g + k] = (z0, z1 of words 0-1; z0, z1 of words 2-3)[k].  V is data in float32.
_PH_M0, _PH_M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_PH_W0, _PH_W1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter: Sequence[np.ndarray], key: Tuple[int, int]) -> List[np.ndarray]:
    """Ten rounds of Philox-4x32: counter = four arrays of 32-bit words, key = two 32-bit words.

    Round: (c0, c1, c2, c3) <- (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1, lo(M0 c0)); the key is
    advanced by the Weyl constants (W0, W1) between rounds.
    """
    c = [np.asarray(x, dtype=np.uint64) & _MASK32 for x in counter]
    k0, k1 = np.uint64(key[0]) & _MASK32, np.uint64(key[1]) & _MASK32
    for _round in range(10):
        p0, p1 = _PH_M0 * c[0], _PH_M1 * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ k0, p1 & _MASK32, (p0 >> np.uint64(32)) ^ c[3] ^ k1, p0 & _MASK32]
        k0, k1 = (k0 + _PH_W0) & _MASK32, (k1 + _PH_W1) & _MASK32
    return c


def _uniform23(x: np.ndarray) -> np.ndarray:
    """(top 23 bits + 0.5) / 2^23: strictly inside (0, 1) and exact in float32 (24 significant bits)."""
    return ((x >> np.uint64(9)).astype(F64) + 0.5) / 8388608.0


def gaussian_V(seed: int, m: int, b: int, r: int) -> np.ndarray:
    """The standard-normal V (b x r) of Alg. 1's t = 0 branch for mode m (0-based), as float32 values."""
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    ng = (r + 3) // 4
    c = np.arange(b, dtype=np.uint64)[:, None]
    g = np.arange(ng, dtype=np.uint64)[None, :]
    shape = (b, ng)
    w = philox4x32_10([np.broadcast_to(c & _MASK32, shape), np.broadcast_to(c >> np.uint64(32), shape),
                       np.broadcast_to(g, shape), np.full(shape, m, dtype=np.uint64)], key)
    u = [_uniform23(x) for x in w]
    V = np.empty((b, ng, 4), dtype=F64)
    for pair in range(2):
        rad = np.sqrt(-2.0 * np.log(u[2 * pair]))
        ang = 2.0 * math.pi * u[2 * pair + 1]
        V[:, :, 2 * pair] = rad * np.cos(ang)
        V[:, :, 2 * pair + 1] = rad * np.sin(ang)
    return V.reshape(b, 4 * ng)[:, :r].astype(np.float32).astype(F64)


def subspace_step_cold(A: np.ndarray, m: int, r: int, seed: int) -> np.ndarray:
    """Alg. 1 at t = 0 for mode m: V i.i.d. standard normal (b_m x r), U = Orthogonalize(A_m V)."""
    Am = unfold(A, m)
    return orthogonalize(Am @ gaussian_V(seed, m, Am.shape[1], r))


def compress_cold(A: np.ndarray, ranks: Sequence[int], seed: int) -> List[np.ndarray]:
    """Alg. 1, t = 0 branch, for every mode of A.  Returns [U_1..U_d]."""
    A = np.asarray(A, dtype=F64)
    return [subspace_step_cold(A, m, int(ranks[m]), seed) for m in range(A.ndim)]


def compress(A: np.ndarray, U_prev: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Alg. 1, warm-start branch, for every mode of A.  Returns [U_1..U_d]."""
    A = np.asarray(A, dtype=F64)
    if len(U_prev) != A.ndim:
        raise ValueError("compress: one previous factor per mode")
    return [subspace_step(A, U_prev[m], m) for m in range(A.ndim)]


def core_project(A: np.ndarray, U: Sequence[np.ndarray]) -> np.ndarray:
    """Core tensor S = A x_1 U_1^T ... x_d U_d^T (Alg. 1's S update; Eq. 3, Eq. 4)."""
    S = np.asarray(A, dtype=F64)
    for m in range(S.ndim):
        S = mode_product(S, np.asarray(U[m], dtype=F64).T, m)
    return S


def reconstruct(S: np.ndarray, U: Sequence[np.ndarray]) -> np.ndarray:
    """Low-rank activation A~ = S x_1 U_1 ... x_d U_d (Eq. 3)."""
    R = np.asarray(S, dtype=F64)
    for m in range(R.ndim):
        R = mode_product(R, np.asarray(U[m], dtype=F64), m)
    return R


def asi(A: np.ndarray, U_prev: Sequence[np.ndarray]) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Whole Alg. 1 (warm-start branch): returns (S, [U_m])."""
    U = compress(A, U_prev)
    return core_project(A, U), U


# --------------------------------------------------------------------------
# Sec. 3.1 Eq. 1: weight gradients (dense definitions)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Conv2dSpec:
    cout: int
    kh: int
    kw: int
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)
    dil: Tuple[int, int] = (1, 1)
    groups: int = 1

    def out_hw(self, H: int, W: int) -> Tuple[int, int]:
        Ho = (H + 2 * self.pad[0] - self.dil[0] * (self.kh - 1) - 1) // self.stride[0] + 1
        Wo = (W + 2 * self.pad[1] - self.dil[1] * (self.kw - 1) - 1) // self.stride[1] + 1
        return Ho, Wo


def _pad_hw(X: np.ndarray, ph: int, pw: int) -> np.ndarray:
    return np.pad(X, [(0, 0)] * (X.ndim - 2) + [(ph, ph), (pw, pw)])


def conv2d_weight_grad_dense(A: np.ndarray, dY: np.ndarray, cs: Conv2dSpec) -> np.ndarray:
    """dL/dW = conv(A, dL/dY) (Eq. 1), cross-correlation convention.

    dW[o,c,kh,kw] = sum_{b,h',w'} dY[b,o,h',w'] *
                    Apad[b, g(o)*C/G + c, h'*s - p + kh*dil, w'*s - p + kw*dil].
    """
    A = np.asarray(A, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    B, C, H, W = A.shape
    Ho, Wo = cs.out_hw(H, W)
    if dY.shape != (B, cs.cout, Ho, Wo):
        raise ValueError(f"dY shape {dY.shape} != {(B, cs.cout, Ho, Wo)}")
    G = cs.groups
    Cg, Og = C // G, cs.cout // G
    Ap = _pad_hw(A, cs.pad[0], cs.pad[1])
    dW = np.zeros((cs.cout, Cg, cs.kh, cs.kw), dtype=F64)
    for kh in range(cs.kh):
        for kw in range(cs.kw):
            h0, w0 = kh * cs.dil[0], kw * cs.dil[1]
            win = Ap[:, :, h0:h0 + cs.stride[0] * (Ho - 1) + 1:cs.stride[0],
                     w0:w0 + cs.stride[1] * (Wo - 1) + 1:cs.stride[1]]      # (B,C,Ho,Wo)
            for g in range(G):
                dW[g * Og:(g + 1) * Og, :, kh, kw] = np.einsum(
                    "bohw,bchw->oc", dY[:, g * Og:(g + 1) * Og], win[:, g * Cg:(g + 1) * Cg])
    return dW


def linear_weight_grad_dense(A: np.ndarray, dY: np.ndarray) -> np.ndarray:
    """Fully-connected analogue of Eq. 1 (Sec. 3.1 footnote): dW[o,d] = sum_{b,n} dY[b,n,o] A[b,n,d]."""
    A = np.asarray(A, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    return np.einsum("bno,bnd->od", dY, A)


# --------------------------------------------------------------------------
# App. A.3 Eq. 14: weight gradient from the compressed form, in the order the
# five cost terms describe.  Each step counts its multiply-accumulates.
# --------------------------------------------------------------------------
def conv2d_weight_grad_lowrank(S, U, dY, cs: Conv2dSpec, count: Optional[dict] = None) -> np.ndarray:
    """Low-rank conv weight gradient following the five terms of C_ASI (Eq. 14).

    1. G1 = dY x_1 U_1^T                       r1 * B * C' * H' * W'  MACs
    2. Z1 = S  x_3 U_3                         r1 * r2 * r3 * r4 * H
    3. Z  = Z1 x_4 U_4                         r1 * r2 * r4 * H * W
    4. T[o,j,kh,kw] = sum_{i,h',w'} G1[i,o,h',w'] Zpad[i,j,..]   r1 * r2 * C' * H' * W' * D^2
    5. dW = T x_j U_2 (per group)              r2 * C' * C * D^2 / groups
    """
    S = np.asarray(S, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    U1, U2, U3, U4 = (np.asarray(u, dtype=F64) for u in U)
    r1, r2, r3, r4 = S.shape
    B, C, H, W = U1.shape[0], U2.shape[0], U3.shape[0], U4.shape[0]
    Ho, Wo = cs.out_hw(H, W)
    macs = {}
    G1 = mode_product(dY, U1.T, 0)                       # (r1, C', H', W')
    macs["G1"] = r1 * B * cs.cout * Ho * Wo
    Z1 = mode_product(S, U3, 2)                          # (r1, r2, H, r4)
    macs["Z1"] = r1 * r2 * r3 * r4 * H
    Z = mode_product(Z1, U4, 3)                          # (r1, r2, H, W)
    macs["Z"] = r1 * r2 * r4 * H * W
    # step 4: a weight-gradient correlation with r1 as batch and r2 as input channels
    T = conv2d_weight_grad_dense(Z, G1, Conv2dSpec(cs.cout, cs.kh, cs.kw, cs.stride, cs.pad, cs.dil, 1))
    macs["T"] = r1 * r2 * cs.cout * Ho * Wo * cs.kh * cs.kw
    # step 5: expand the r2 axis back to the input channels of each output channel's group
    G = cs.groups
    Cg, Og = C // G, cs.cout // G
    dW = np.zeros((cs.cout, Cg, cs.kh, cs.kw), dtype=F64)
    for g in range(G):
        dW[g * Og:(g + 1) * Og] = np.einsum("ojhw,cj->ochw", T[g * Og:(g + 1) * Og], U2[g * Cg:(g + 1) * Cg])
    macs["dW"] = r2 * cs.cout * Cg * cs.kh * cs.kw
    if count is not None:
        count.update(macs)
    return dW


def linear_weight_grad_lowrank(S, U, dY, count: Optional[dict] = None) -> np.ndarray:
    """Low-rank linear weight gradient: the conv order of Eq. 14 carried to a 3-mode tensor.

    1. G1[i,n,o] = sum_b U_1[b,i] dY[b,n,o]
    2. G2[i,j,o] = sum_n U_2[n,j] G1[i,n,o]
    3. T[o,k]    = sum_{i,j} G2[i,j,o] S[i,j,k]
    4. dW[o,d]   = sum_k T[o,k] U_3[d,k]
    """
    S = np.asarray(S, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    U1, U2, U3 = (np.asarray(u, dtype=F64) for u in U)
    r1, r2, r3 = S.shape
    B, N, D = U1.shape[0], U2.shape[0], U3.shape[0]
    Do = dY.shape[2]
    G1 = mode_product(dY, U1.T, 0)
    G2 = mode_product(G1, U2.T, 1)
    T = np.einsum("ijo,ijk->ok", G2, S)
    dW = T @ U3.T
    if count is not None:
        count.update({"G1": r1 * B * N * Do, "G2": r1 * r2 * N * Do, "T": r1 * r2 * r3 * Do, "dW": r3 * Do * D})
    return dW


# --------------------------------------------------------------------------
# Cost model (Eq. 5, Eq. 10, App. A Eq. 11-18).  Unit: multiply-accumulates.
# --------------------------------------------------------------------------
def storage_elements(dims: Sequence[int], ranks: Sequence[int]) -> int:
    """M_i = prod r_m + sum D_m r_m (Eq. 5)."""
    return math.prod(ranks) + sum(d * r for d, r in zip(dims, ranks))


def overhead_asi(dims: Sequence[int], ranks: Sequence[int]) -> int:
    """O_ASI = sum_m (2 d d' r_m + r_m^3) (Eq. 13), d' = product of the other dims."""
    tot = math.prod(dims)
    return sum(2 * tot * r + r ** 3 for r in ranks)


def overhead_hosvd(dims: Sequence[int]) -> int:
    """O_HOSVD = sum_d max(d,P_d)^2 min(d,P_d) (Eq. 10)."""
    tot = math.prod(dims)
    return sum(max(d, tot // d) ** 2 * min(d, tot // d) for d in dims)


def cost_asi_backward(dims, ranks, cout: int, Ho: int, Wo: int, D: int) -> int:
    """C_ASI (Eq. 14) for a D x D convolution with groups = 1."""
    B, C, H, W = dims
    r1, r2, r3, r4 = ranks
    return (r1 * B * cout * Ho * Wo + r1 * r2 * r3 * r4 * H + r1 * r2 * r4 * H * W
            + r1 * r2 * cout * Ho * Wo * D * D + r2 * cout * C * D * D)


def cost_vanilla_backward(dims, cout: int, Ho: int, Wo: int, D: int) -> int:
    """C_vanilla = D^2 C C' B H' W' (Eq. 15)."""
    B, C, H, W = dims
    return D * D * C * cout * B * Ho * Wo


def cost_vanilla_forward(dims, cout: int, D: int) -> int:
    """O_vanilla = D^2 C C' B H W (Eq. 16; the paper writes it with the input H, W)."""
    B, C, H, W = dims
    return D * D * C * cout * B * H * W


def speedup_ratio(dims, ranks, cout: int, Ho: int, Wo: int, D: int) -> float:
    """R_S (Eq. 17)."""
    ov = cost_vanilla_forward(dims, cout, D)
    return (ov + cost_vanilla_backward(dims, cout, Ho, Wo, D)) / (
        ov + overhead_asi(dims, ranks) + cost_asi_backward(dims, ranks, cout, Ho, Wo, D))


def compression_ratio(dims, ranks) -> float:
    """R_C (Eq. 18)."""
    return math.prod(dims) / storage_elements(dims, ranks)


# --------------------------------------------------------------------------
# helpers used by the parity tests (definitions, not method steps)
# --------------------------------------------------------------------------
def projector(U: np.ndarray) -> np.ndarray:
    """Orthogonal projector U U^T onto range(U) - the unique part of a factor."""
    U = np.asarray(U, dtype=F64)
    return U @ U.T


def max_rel_err(x: np.ndarray, ref: np.ndarray) -> float:
    """max|x - ref| / max|ref| - the error measure of the parity bar."""
    x = np.asarray(x, dtype=F64)
    ref = np.asarray(ref, dtype=F64)
    den = float(np.max(np.abs(ref)))
    num = float(np.max(np.abs(x - ref))) if x.size else 0.0
    if not np.isfinite(num):
        return float("inf")
    return num / den if den > 0 else num
