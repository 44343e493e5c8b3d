"""Pins for the float64 oracle: facts fixed by the paper or by mathematics.

Each test would fail on a plausible mistake in the oracle (dropped term, wrong
sign or index, transposed operand).  None of them re-types the oracle's own
formula: they use brute-force loops on tiny inputs, closed forms, invariants,
LAPACK routines for special cases, and cells the paper prints.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import asi_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_table_cells.txt")


def _rng(seed):
    return np.random.default_rng(seed)


def _orth(rng, n, r):
    q, _ = np.linalg.qr(rng.standard_normal((n, r)))
    return q


# ---------------------------------------------------------------- unfold / mode product
def test_unfold_brute_force():
    rng = _rng(1)
    A = rng.standard_normal((3, 4, 2, 5))
    for m in range(4):
        Am = O.unfold(A, m)
        assert Am.shape == (A.shape[m], A.size // A.shape[m])
        others = [k for k in range(4) if k != m]
        col = 0
        for idx in itertools.product(*[range(A.shape[k]) for k in others]):
            for i in range(A.shape[m]):
                full = [0] * 4
                full[m] = i
                for k, v in zip(others, idx):
                    full[k] = v
                assert Am[i, col] == A[tuple(full)]
            col += 1


def test_mode_product_brute_force_eq4():
    """Eq. 4 with B of shape (Q, P_m), nested loops, non-square shapes."""
    rng = _rng(2)
    G = rng.standard_normal((3, 4, 2, 5))
    for m in range(4):
        Q = 6 if m != 1 else 3
        Bm = rng.standard_normal((Q, G.shape[m]))
        R = O.mode_product(G, Bm, m)
        shp = list(G.shape)
        shp[m] = Q
        assert R.shape == tuple(shp)
        for idx in itertools.product(*[range(s) for s in shp]):
            acc = 0.0
            for p in range(G.shape[m]):
                src = list(idx)
                src[m] = p
                acc += G[tuple(src)] * Bm[idx[m], p]
            assert abs(R[idx] - acc) < 1e-12


def test_mode_products_commute_all_orders():
    rng = _rng(3)
    A = rng.standard_normal((5, 6, 4, 7))
    U = [_orth(rng, n, r) for n, r in zip(A.shape, (2, 3, 2, 4))]
    S = O.core_project(A, U)
    for order in itertools.permutations(range(4)):
        T = A
        for m in order:
            T = O.mode_product(T, U[m].T, m)
        assert np.max(np.abs(T - S)) < 1e-12


def test_core_brute_force_definition():
    rng = _rng(4)
    dims, ranks = (3, 4, 2, 5), (2, 3, 2, 2)
    A = rng.standard_normal(dims)
    U = [rng.standard_normal((n, r)) for n, r in zip(dims, ranks)]   # need not be orthonormal
    S = O.core_project(A, U)
    for q in itertools.product(*[range(r) for r in ranks]):
        acc = 0.0
        for p in itertools.product(*[range(n) for n in dims]):
            w = A[p]
            for m in range(4):
                w *= U[m][p[m], q[m]]
            acc += w
        assert abs(S[q] - acc) < 1e-11
    # reconstruction is the adjoint: <reconstruct(S'), A> = <S', core(A)>
    S2 = rng.standard_normal(ranks)
    assert abs(np.sum(O.reconstruct(S2, U) * A) - np.sum(S2 * S)) < 1e-10


# ---------------------------------------------------------------- orthogonalisation
@pytest.mark.parametrize("n,r", [(7, 5), (64, 16), (40, 40), (3, 1)])
def test_orthogonalize_is_positive_diag_qr(n, r):
    rng = _rng(10 + n)
    P = rng.standard_normal((n, r)) * (np.arange(1, r + 1) ** -3.0)   # badly scaled columns
    Q = O.orthogonalize(P)
    assert np.max(np.abs(Q.T @ Q - np.eye(r))) < 1e-13
    R = Q.T @ P
    assert np.all(np.diag(R) > 0)
    assert np.max(np.abs(np.tril(R, -1))) < 1e-12 * np.max(np.abs(R))
    assert np.max(np.abs(Q @ R - P)) < 1e-13 * np.max(np.abs(P))
    # LAPACK's Householder QR, columns sign-fixed, is the same unique factor
    q2, r2 = np.linalg.qr(P)
    q2 = q2 * np.sign(np.diag(r2))
    assert np.max(np.abs(Q - q2)) < 1e-9


def test_orthogonalize_ill_conditioned_stays_orthonormal():
    rng = _rng(11)
    U, _ = np.linalg.qr(rng.standard_normal((50, 12)))
    W, _ = np.linalg.qr(rng.standard_normal((12, 12)))
    P = (U * np.logspace(0, -9, 12)) @ W.T
    Q = O.orthogonalize(P)
    assert np.max(np.abs(Q.T @ Q - np.eye(12))) < 1e-13
    # same range as P
    assert np.max(np.abs(U @ (U.T @ Q) - Q)) < 1e-6


def test_orthogonalize_breakdown():
    rng = _rng(12)
    P = rng.standard_normal((9, 4))
    P[:, 2] = 2.0 * P[:, 0] - P[:, 1]
    with pytest.raises(O.OrthogonalizeBreakdown) as e:
        O.orthogonalize(P)
    assert e.value.column == 2
    with pytest.raises(O.OrthogonalizeBreakdown):
        O.orthogonalize(np.zeros((5, 2)))


# ---------------------------------------------------------------- subspace step
def test_subspace_P_equals_gram_times_basis_and_ignores_column_order():
    rng = _rng(20)
    A = rng.standard_normal((4, 5, 3, 6))
    for m in range(4):
        Up = _orth(rng, A.shape[m], 2)
        Am = np.moveaxis(A, m, 0).reshape(A.shape[m], -1)
        gram = np.zeros((A.shape[m], A.shape[m]))
        for c in rng.permutation(Am.shape[1]):          # any column order, explicit outer products
            gram += np.outer(Am[:, c], Am[:, c])
        assert np.max(np.abs(O.subspace_P(A, Up, m) - gram @ Up)) < 1e-11


def test_full_rank_reconstructs_exactly():
    rng = _rng(21)
    A = rng.standard_normal((4, 5, 3, 6))
    Up = [rng.standard_normal((n, n)) for n in A.shape]      # any full-rank start
    S, U = O.asi(A, Up)
    assert S.shape == A.shape
    assert np.max(np.abs(O.reconstruct(S, U) - A)) < 1e-12
    A3 = rng.standard_normal((5, 7, 4))
    S3, U3 = O.asi(A3, [rng.standard_normal((n, n)) for n in A3.shape])
    assert np.max(np.abs(O.reconstruct(S3, U3) - A3)) < 1e-12


def test_factors_orthonormal_positive_diag():
    rng = _rng(22)
    A = rng.standard_normal((6, 8, 5, 5))
    ranks = (3, 4, 2, 5)
    Up = [_orth(rng, n, r) for n, r in zip(A.shape, ranks)]
    U = O.compress(A, Up)
    for m, (u, r) in enumerate(zip(U, ranks)):
        assert u.shape == (A.shape[m], r)
        assert np.max(np.abs(u.T @ u - np.eye(r))) < 1e-13
        assert np.all(np.diag(u.T @ O.subspace_P(A, Up[m], m)) > 0)


def _sin_theta(U, V):
    """Largest principal-angle sine between range(U) and range(V) (orthonormal bases)."""
    return np.linalg.norm(V - U @ (U.T @ V), 2)


def test_planted_gap_converges_to_svd_subspace_at_textbook_rate():
    rng = _rng(23)
    n, b, r, gamma = 12, 40, 4, 3.0
    Ul, _ = np.linalg.qr(rng.standard_normal((n, n)))
    Wr, _ = np.linalg.qr(rng.standard_normal((b, n)))
    sig = np.concatenate([np.linspace(2.0, 1.0, r), np.linspace(1.0 / gamma, 0.05, n - r)])
    M = (Ul * sig) @ Wr.T
    A = M.reshape(n, 5, 8)                       # mode-0 unfolding of a 3-mode tensor is M
    Uk = _orth(rng, n, r)
    u_svd = np.linalg.svd(M)[0][:, :r]           # LAPACK
    assert np.max(np.abs(u_svd @ u_svd.T - Ul[:, :r] @ Ul[:, :r].T)) < 1e-10
    c = Ul[:, :r].T @ Uk
    tan0 = np.linalg.norm((Ul[:, r:].T @ Uk) @ np.linalg.inv(c), 2)
    errs = []
    for k in range(1, 9):
        Uk = O.subspace_step(A, Uk, 0)
        s = _sin_theta(u_svd, Uk)
        errs.append(s)
        assert s <= gamma ** (-2 * k) * tan0 * (1 + 1e-9) + 1e-13
    assert errs[-1] < 1e-6 and errs[-1] < errs[0]
    # the rate is really gamma^-2 per step, not gamma^-1 (one step = one product with A A^T)
    assert errs[3] / errs[2] < 1.3 * gamma ** -2


def test_warm_start_uses_current_activation_and_previous_basis():
    """One step from the exact basis of a rank-r unfolding returns that basis' range."""
    rng = _rng(24)
    A, fac = _exact_tucker(rng, (5, 6, 4, 7), (2, 3, 2, 3))
    for m in range(4):
        Up = _orth(rng, A.shape[m], A.shape[m])[:, :fac[m].shape[1]]   # generic start
        U = O.subspace_step(A, Up, m)
        assert _sin_theta(fac[m], U) < 1e-10


def _exact_tucker(rng, dims, ranks):
    fac = [_orth(rng, n, r) for n, r in zip(dims, ranks)]
    x = rng.standard_normal(ranks)
    for m, f in enumerate(fac):
        x = np.moveaxis(np.tensordot(f, x, axes=([1], [m])), 0, m)
    return x, fac


# ---------------------------------------------------------------- projection invariants
def test_pythagoras_of_orthogonal_projection():
    rng = _rng(30)
    A = rng.standard_normal((6, 7, 5, 4))
    Up = [_orth(rng, n, r) for n, r in zip(A.shape, (3, 3, 2, 2))]
    S, U = O.asi(A, Up)
    Ah = O.reconstruct(S, U)
    nA, nS, nR = np.sum(A * A), np.sum(S * S), np.sum((A - Ah) ** 2)
    assert abs(nA - nS - nR) < 1e-11 * nA
    assert abs(np.sum(Ah * Ah) - nS) < 1e-11 * nA
    assert nR > 1e-3 * nA                         # the case is not trivially exact


# ---------------------------------------------------------------- dense weight gradients
def _naive_conv_dw(A, dY, cout, kh, kw, s, p, d, groups):
    B, C, H, W = A.shape
    Ho, Wo = dY.shape[2], dY.shape[3]
    Cg, Og = C // groups, cout // groups
    dW = np.zeros((cout, Cg, kh, kw))
    for o in range(cout):
        g = o // Og
        for c in range(Cg):
            for a in range(kh):
                for e in range(kw):
                    acc = 0.0
                    for b in range(B):
                        for y in range(Ho):
                            for x in range(Wo):
                                hh = y * s[0] - p[0] + a * d[0]
                                ww = x * s[1] - p[1] + e * d[1]
                                if 0 <= hh < H and 0 <= ww < W:
                                    acc += dY[b, o, y, x] * A[b, g * Cg + c, hh, ww]
                    dW[o, c, a, e] = acc
    return dW


CONV_CASES = [
    # C, cout, H, W, kh, kw, stride, pad, dil, groups
    (3, 4, 6, 5, 3, 3, (1, 1), (1, 1), (1, 1), 1),
    (4, 4, 7, 6, 3, 3, (2, 2), (0, 0), (1, 1), 1),
    (4, 6, 7, 7, 3, 2, (2, 1), (1, 0), (1, 2), 2),
    (4, 4, 5, 5, 3, 3, (1, 1), (1, 1), (1, 1), 4),      # depthwise
    (3, 5, 4, 4, 1, 1, (1, 1), (0, 0), (1, 1), 1),      # pointwise
    (2, 2, 8, 8, 3, 3, (1, 1), (2, 2), (2, 2), 1),      # dilated
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_dw_dense_vs_seven_loops(case):
    C, cout, H, W, kh, kw, s, p, d, g = case
    rng = _rng(40)
    cs = O.Conv2dSpec(cout, kh, kw, s, p, d, g)
    Ho, Wo = cs.out_hw(H, W)
    A = rng.standard_normal((2, C, H, W))
    dY = rng.standard_normal((2, cout, Ho, Wo))
    ref = _naive_conv_dw(A, dY, cout, kh, kw, s, p, d, g)
    assert np.max(np.abs(O.conv2d_weight_grad_dense(A, dY, cs) - ref)) < 1e-12


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_dw_dense_vs_autograd_library(case):
    """Eq. 1 is what a library's conv2d backward computes (float64 autograd on the CPU)."""
    torch = pytest.importorskip("torch")
    C, cout, H, W, kh, kw, s, p, d, g = case
    rng = _rng(41)
    cs = O.Conv2dSpec(cout, kh, kw, s, p, d, g)
    Ho, Wo = cs.out_hw(H, W)
    A = rng.standard_normal((3, C, H, W))
    dY = rng.standard_normal((3, cout, Ho, Wo))
    w = torch.zeros((cout, C // g, kh, kw), dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.conv2d(torch.from_numpy(A), w, None, s, p, d, g)
    assert tuple(y.shape) == dY.shape
    y.backward(torch.from_numpy(dY))
    assert np.max(np.abs(O.conv2d_weight_grad_dense(A, dY, cs) - w.grad.numpy())) < 1e-12


def test_linear_dw_dense_brute_force_and_equals_pointwise_conv():
    rng = _rng(42)
    B, N, D, Do = 2, 3, 4, 5
    A = rng.standard_normal((B, N, D))
    dY = rng.standard_normal((B, N, Do))
    ref = np.zeros((Do, D))
    for o in range(Do):
        for dd in range(D):
            for b in range(B):
                for n in range(N):
                    ref[o, dd] += dY[b, n, o] * A[b, n, dd]
    assert np.max(np.abs(O.linear_weight_grad_dense(A, dY) - ref)) < 1e-13
    # a 1x1 convolution over (B, D, N, 1) maps is the same contraction
    A4 = np.transpose(A, (0, 2, 1))[..., None]
    dY4 = np.transpose(dY, (0, 2, 1))[..., None]
    dw4 = O.conv2d_weight_grad_dense(A4, dY4, O.Conv2dSpec(Do, 1, 1))
    assert np.max(np.abs(dw4[:, :, 0, 0] - ref)) < 1e-13


# ---------------------------------------------------------------- low-rank weight gradients
@pytest.mark.parametrize("case", CONV_CASES)
def test_lowrank_conv_dw_equals_dense_dw_of_reconstruction(case):
    """For ANY core and factors (linearity) - pins Eq. 14's order independently of compress."""
    C, cout, H, W, kh, kw, s, p, d, g = case
    rng = _rng(50)
    B = 3
    ranks = (2, min(3, C), 3, 2)
    S = rng.standard_normal(ranks)
    U = [rng.standard_normal((n, r)) for n, r in zip((B, C, H, W), ranks)]
    cs = O.Conv2dSpec(cout, kh, kw, s, p, d, g)
    Ho, Wo = cs.out_hw(H, W)
    dY = rng.standard_normal((B, cout, Ho, Wo))
    cnt = {}
    lr = O.conv2d_weight_grad_lowrank(S, U, dY, cs, cnt)
    ref = _naive_conv_dw(O.reconstruct(S, U), dY, cout, kh, kw, s, p, d, g)
    assert np.max(np.abs(lr - ref)) < 1e-11 * max(1.0, np.max(np.abs(ref)))
    if g == 1 and kh == kw:
        assert sum(cnt.values()) == O.cost_asi_backward((B, C, H, W), ranks, cout, Ho, Wo, kh)


def test_lowrank_linear_dw_equals_dense_dw_of_reconstruction():
    rng = _rng(51)
    dims, ranks, Do = (4, 5, 6), (2, 3, 4), 7
    S = rng.standard_normal(ranks)
    U = [rng.standard_normal((n, r)) for n, r in zip(dims, ranks)]
    dY = rng.standard_normal((dims[0], dims[1], Do))
    cnt = {}
    lr = O.linear_weight_grad_lowrank(S, U, dY, cnt)
    Ah = O.reconstruct(S, U)
    ref = np.zeros((Do, dims[2]))
    for b in range(dims[0]):
        ref += dY[b].T @ Ah[b]
    assert np.max(np.abs(lr - ref)) < 1e-11
    # all four terms of the derived cost, as integers worked out by hand for this shape:
    # r1 B N Do = 2*4*5*7, r1 r2 N Do = 2*3*5*7, r1 r2 r3 Do = 2*3*4*7, r3 Do D = 4*7*6
    assert cnt == {"G1": 280, "G2": 210, "T": 168, "dW": 168}


def test_exact_tucker_compressed_dw_equals_dense_dw():
    """Exactly-Tucker activation: one step from a generic basis loses nothing."""
    rng = _rng(52)
    dims, ranks = (4, 6, 5, 5), (2, 3, 2, 3)
    A, _ = _exact_tucker(rng, dims, ranks)
    Up = [_orth(rng, n, r) for n, r in zip(dims, ranks)]
    S, U = O.asi(A, Up)
    assert np.max(np.abs(O.reconstruct(S, U) - A)) < 1e-11
    cs = O.Conv2dSpec(4, 3, 3, (1, 1), (1, 1))
    dY = rng.standard_normal((4, 4, 5, 5))
    dense = _naive_conv_dw(A, dY, 4, 3, 3, (1, 1), (1, 1), (1, 1), 1)
    assert np.max(np.abs(O.conv2d_weight_grad_lowrank(S, U, dY, cs) - dense)) < 1e-10


# ---------------------------------------------------------------- cost model vs printed cells
def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v, _unit, _cite = [s.strip() for s in line.split("|")]
            out[k] = float(v)
    return out


MIB = 1024.0 * 1024.0
# inputs of the last convolutions, counted from the network's end
RESNET18_TAIL = [  # (C, H, W, cout, D, Ho, Wo)
    (512, 7, 7, 512, 3, 7, 7), (512, 7, 7, 512, 3, 7, 7),
    (256, 14, 14, 512, 1, 7, 7),            # the 1x1 stride-2 shortcut of the last stage
    (512, 7, 7, 512, 3, 7, 7)]
MOBILENETV2_TAIL = [(320, 7, 7), (960, 7, 7), (960, 7, 7), (160, 7, 7)]


def test_cost_model_reproduces_printed_cells():
    g = _golden()
    for B, tag in ((64, "b64"), (128, "b128")):
        for k in (2, 4):
            mem = sum(B * C * H * W * 4 for C, H, W, *_ in RESNET18_TAIL[:k]) / MIB
            assert abs(mem - g[f"resnet18_{tag}_{k}layers_mem"]) < 0.006
            mem = sum(B * C * H * W * 4 for C, H, W in MOBILENETV2_TAIL[:k]) / MIB
            assert abs(mem - g[f"mobilenetv2_{tag}_{k}layers_mem"]) < 0.006
    for k in (2, 4):
        macs = 0
        for C, H, W, cout, D, Ho, Wo in RESNET18_TAIL[:k]:
            dims = (64, C, H, W)
            macs += O.cost_vanilla_forward(dims, cout, D) + O.cost_vanilla_backward(dims, cout, Ho, Wo, D)
        assert abs(macs / 1e9 - g[f"resnet18_b64_{k}layers_gflops"]) < 0.006   # "FLOPs" are MACs


def test_cost_closed_forms():
    dims, ranks = (64, 512, 7, 7), (16, 48, 5, 5)
    assert O.storage_elements(dims, ranks) == 16 * 48 * 25 + 64 * 16 + 512 * 48 + 35 + 35 == 44870
    tot = 64 * 512 * 49
    assert O.overhead_asi(dims, ranks) == 2 * tot * (16 + 48 + 5 + 5) + 16 ** 3 + 48 ** 3 + 2 * 125
    assert abs(O.compression_ratio(dims, ranks) - tot / 44870) < 1e-12
    # all ranks 1 (the paper's Fig. 2 setting): R_C = BCHW / (1 + B + C + H + W)
    assert abs(O.compression_ratio(dims, (1, 1, 1, 1)) - tot / (1 + 64 + 512 + 14)) < 1e-12
    assert O.overhead_hosvd((2, 3, 4, 5)) == 60 ** 2 * 2 + 40 ** 2 * 3 + 30 ** 2 * 4 + 24 ** 2 * 5
    c = O.cost_asi_backward(dims, ranks, 512, 7, 7, 3)
    assert c == 16 * 64 * 512 * 49 + 16 * 48 * 25 * 7 + 16 * 48 * 5 * 49 + 16 * 48 * 512 * 49 * 9 + 48 * 512 * 512 * 9
    ov, cv = O.cost_vanilla_forward(dims, 512, 3), O.cost_vanilla_backward(dims, 512, 7, 7, 3)
    assert ov == cv == 9 * 512 * 512 * 64 * 49
    rs = O.speedup_ratio(dims, ranks, 512, 7, 7, 3)
    assert 1.0 < rs < 2.0


def test_speedup_ratio_against_hand_expanded_integers():
    """R_S (Eq. 17) on a shape small enough to expand every term of Eq. 13-16 by hand.

    dims (B,C,H,W) = (2,3,4,5), ranks (1,2,2,3), 3x3 convolution to C' = 4 with H' x W' = 4 x 5:
      O_vanilla = D^2 C C' B H W   = 9*3*4*2*4*5                                  = 4320
      C_vanilla = D^2 C C' B H' W' = 9*3*4*2*4*5                                  = 4320
      O_ASI     = sum_m (2*120*r_m + r_m^3) = 240*(1+2+2+3) + (1+8+8+27)          = 1964
      C_ASI     = 1*2*4*20 + 1*2*2*3*4 + 1*2*3*4*5 + 1*2*4*20*9 + 2*4*3*9
                = 160 + 48 + 120 + 1440 + 216                                     = 1984
      R_S = (4320 + 4320) / (4320 + 1964 + 1984) = 8640 / 8268
    A wrong or missing term in numerator or denominator changes the literal quotient."""
    dims, ranks = (2, 3, 4, 5), (1, 2, 2, 3)
    assert O.cost_vanilla_forward(dims, 4, 3) == 4320
    assert O.cost_vanilla_backward(dims, 4, 4, 5, 3) == 4320
    assert O.overhead_asi(dims, ranks) == 1964
    assert O.cost_asi_backward(dims, ranks, 4, 4, 5, 3) == 1984
    assert abs(O.speedup_ratio(dims, ranks, 4, 4, 5, 3) - 8640.0 / 8268.0) < 1e-15
    # H' W' differs from H W (stride 2): only C_vanilla and C_ASI's terms 1 and 4 change
    #   C_vanilla = 9*3*4*2*2*3 = 1296;  C_ASI = 1*2*4*6 + 48 + 120 + 1*2*4*6*9 + 216 = 48+48+120+432+216 = 864
    assert abs(O.speedup_ratio(dims, ranks, 4, 2, 3, 3) - (4320.0 + 1296.0) / (4320.0 + 1964.0 + 864.0)) < 1e-15


def test_max_rel_err_on_hand_made_arrays():
    """The yardstick of every parity assert: max|x - ref| / max|ref| (not elementwise, not Frobenius)."""
    ref = np.array([[1.0, -4.0], [0.0, 2.0]])
    x = np.array([[1.5, -4.0], [0.25, 1.0]])
    assert O.max_rel_err(x, ref) == 1.0 / 4.0                     # largest difference 1.0 (last entry), largest |ref| 4
    assert O.max_rel_err(ref, ref) == 0.0
    assert O.max_rel_err(ref, x) == 1.0 / 4.0                     # max|x| is 4 as well
    assert O.max_rel_err(2.0 * ref, ref) == 1.0
    # an error on a zero entry of the reference still counts against the largest entry (no division by zero)
    assert O.max_rel_err(np.array([0.0, 0.5]), np.array([0.0, 0.0])) == 0.5     # zero reference: absolute error
    assert O.max_rel_err(np.array([1e-3, 10.0]), np.array([0.0, 10.0])) == 1e-4
    # non-finite results never pass a bar
    assert O.max_rel_err(np.array([np.nan, 1.0]), np.array([1.0, 1.0])) == float("inf")
    assert O.max_rel_err(np.array([np.inf, 1.0]), np.array([1.0, 1.0])) == float("inf")
    assert O.max_rel_err(np.array([-np.inf]), np.array([1.0])) == float("inf")
    # float32 inputs are compared in float64
    assert O.max_rel_err(np.array([1.0], dtype=np.float32), np.array([1.0 + 1e-12])) < 2e-12


def test_projector_is_the_orthogonal_projector():
    rng = _rng(77)
    U = _orth(rng, 7, 3)
    Pm = O.projector(U)
    assert Pm.shape == (7, 7)
    assert np.max(np.abs(Pm @ Pm - Pm)) < 1e-13 and np.max(np.abs(Pm - Pm.T)) < 1e-15
    assert abs(np.trace(Pm) - 3.0) < 1e-13
    # invariant under a rotation and sign change of the basis
    R, _ = np.linalg.qr(rng.standard_normal((3, 3)))
    assert np.max(np.abs(O.projector(U @ R) - Pm)) < 1e-13
    # elementwise against the definition
    for i in range(7):
        for j in range(7):
            assert abs(Pm[i, j] - sum(U[i, k] * U[j, k] for k in range(3))) < 1e-15


# ---------------------------------------------------------------- Alg. 1, t = 0: the Gaussian draw
def test_philox4x32_10_known_answers():
    """The known-answer vectors distributed with the published generator (tests/golden/philox4x32_10_kat.txt)."""
    rows = [ln.split() for ln in open(os.path.join(os.path.dirname(GOLDEN), "philox4x32_10_kat.txt")) if ln.strip() and ln[0] != "#"]
    assert len(rows) == 3
    kat = [(tuple(int(x, 16) for x in r[0:4]), tuple(int(x, 16) for x in r[4:6]), tuple(int(x, 16) for x in r[6:10]))
           for r in rows]
    for ctr, key, want in kat:
        got = O.philox4x32_10([np.array([c], dtype=np.uint64) for c in ctr], key)
        assert tuple(int(x[0]) for x in got) == want
    # vectorised over counters: every lane equals its own scalar call
    c0 = np.array([0, 0xffffffff, 0x243f6a88, 7], dtype=np.uint64)
    got = O.philox4x32_10([c0, c0 * 0 + 5, c0 * 0, c0 * 0 + 2], (11, 12))
    for lane in range(4):
        one = O.philox4x32_10([c0[lane:lane + 1], np.array([5], dtype=np.uint64), np.array([0], dtype=np.uint64),
                               np.array([2], dtype=np.uint64)], (11, 12))
        assert [int(x[lane]) for x in got] == [int(x[0]) for x in one]


def test_gaussian_V_is_standard_normal_and_counter_addressed():
    V = O.gaussian_V(seed=0x0123456789abcdef, m=1, b=200000, r=6)
    assert V.shape == (200000, 6) and V.dtype == np.float64
    assert np.array_equal(V, V.astype(np.float32).astype(np.float64))            # float32 data
    # moments of N(0, 1): mean 0, variance 1, skewness 0, kurtosis 3 (1.2M samples: 5 sigma bounds)
    x = V.ravel()
    n = x.size
    assert abs(x.mean()) < 5 / np.sqrt(n)
    assert abs(x.var() - 1.0) < 5 * np.sqrt(2.0 / n)
    assert abs(np.mean(x ** 3)) < 5 * np.sqrt(15.0 / n)
    assert abs(np.mean(x ** 4) - 3.0) < 5 * np.sqrt(96.0 / n)
    # tail mass beyond 3 sigma: 0.0027
    assert abs(np.mean(np.abs(x) > 3.0) - 0.0026998) < 5 * np.sqrt(0.0027 / n)
    # columns and rows are uncorrelated
    C = np.corrcoef(V.T)
    assert np.max(np.abs(C - np.eye(6))) < 5 / np.sqrt(200000)
    assert abs(np.corrcoef(V[:-1, 0], V[1:, 0])[0, 1]) < 5 / np.sqrt(200000)
    # counter addressing: an entry depends only on (seed, mode, column, rank column), not on b or r
    W = O.gaussian_V(seed=0x0123456789abcdef, m=1, b=1000, r=3)
    assert np.array_equal(W, V[:1000, :3])
    assert not np.array_equal(O.gaussian_V(0x0123456789abcdef, 2, 1000, 3), W)      # another mode: another stream
    assert not np.array_equal(O.gaussian_V(0x0123456789abcdee, 1, 1000, 3), W)      # another seed
    # Box-Muller by hand for one entry: words -> 23-bit uniforms -> (radius, angle)
    w = O.philox4x32_10([np.array([5], dtype=np.uint64), np.array([0], dtype=np.uint64), np.array([0], dtype=np.uint64),
                         np.array([1], dtype=np.uint64)], (0x89abcdef, 0x01234567))
    u1 = ((int(w[0][0]) >> 9) + 0.5) / 2 ** 23
    u2 = ((int(w[1][0]) >> 9) + 0.5) / 2 ** 23
    z0 = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    z1 = np.sqrt(-2.0 * np.log(u1)) * np.sin(2.0 * np.pi * u2)
    assert V[5, 0] == np.float32(z0) and V[5, 1] == np.float32(z1)


def test_cold_start_step_finds_the_range_of_an_exactly_low_rank_unfolding():
    """t = 0 branch of Alg. 1: for an unfolding of exact rank r, range(A_m V) = range(A_m) for any V of
    full column rank, so one cold step already gives the SVD's subspace; on a planted spectral gap the
    cold step is at a finite angle and the warm steps that follow converge at the rate gamma^-2."""
    rng = _rng(61)
    dims, ranks = (5, 7, 6, 4), (2, 3, 2, 2)
    A, Ut = _exact_tucker(rng, dims, ranks)
    U = O.compress_cold(A, ranks, seed=2025)
    for m in range(4):
        assert np.max(np.abs(U[m].T @ U[m] - np.eye(ranks[m]))) < 1e-13
        lead = np.linalg.svd(O.unfold(A, m), full_matrices=False)[0][:, :ranks[m]]
        assert np.max(np.abs(O.projector(U[m]) - O.projector(lead))) < 1e-10
    # the definition written out for one mode: U = Q of A_m V with V from the generator
    Am = O.unfold(A, 1)
    Q, R = np.linalg.qr(Am @ O.gaussian_V(2025, 1, Am.shape[1], 3))
    assert np.max(np.abs(U[1] - Q * np.sign(np.diag(R)))) < 1e-12
    # planted gap: tan(theta) shrinks by at least gamma^-2 per warm step after the cold one
    n, b, r, gamma = 12, 40, 3, 4.0
    Qa = _orth(rng, n, n)
    Qb = _orth(rng, b, n)
    sv = np.array([3.0, 2.5, 2.0] + [2.0 / gamma] * (n - r))
    M = (Qa * sv) @ Qb.T
    U0 = O.subspace_step_cold(M, 0, r, seed=7)
    errs = []
    Uk = U0
    for _ in range(4):
        errs.append(np.linalg.norm(Qa[:, r:].T @ Uk @ np.linalg.inv(Qa[:, :r].T @ Uk), 2))
        Uk = O.subspace_step(M, Uk, 0)
    assert errs[0] > 1e-2 and all(e1 <= e0 * gamma ** -2 * (1 + 1e-9) for e0, e1 in zip(errs, errs[1:]))
