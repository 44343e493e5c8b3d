"""GPU parity: the HIP path (through the C ABI) against the float64 oracle on the
same seeded inputs.  Factors are compared through their projectors U U^T (the
unique part); core and weight gradient are compared teacher-forced (same U, S
on both sides) and end to end.

Bar: max|x - ref| / max|ref| <= 1e-4 for fp32 inputs, 2e-2 for bf16 inputs with
fp32 accumulation.
"""
import numpy as np
import pytest
import torch

from asi_inputs import CONFIGS, LayerStream
from asi_inputs.configs import Layer
from oracle import asi_oracle as O

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
F64 = np.float64


def _runner(layer):
    from paper_2505_05086_amd.runner import LayerRunner
    return LayerRunner(layer)


def _conv_spec(lay):
    return O.Conv2dSpec(lay.cout, lay.k, lay.k, (lay.stride,) * 2, (lay.pad,) * 2, (lay.dil,) * 2, lay.groups)


def _oracle_dw(lay, S, U, dY):
    if lay.kind == "conv2d":
        return O.conv2d_weight_grad_lowrank(S, U, dY, _conv_spec(lay))
    return O.linear_weight_grad_lowrank(S, U, dY)


def _np(t):
    return t.detach().float().cpu().numpy().astype(F64)


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def check_compress(run, lay, A_np, Uprev_np, tol, tag):
    """One warm-started step on both sides from the same previous factors."""
    A64 = A_np.astype(F64)
    U_or = O.compress(A64, [u.astype(F64) for u in Uprev_np])
    run.set_factors(Uprev_np)
    A_t = run.upload(A_np)
    U_gpu = run.compress(A_t)
    torch.cuda.synchronize()
    assert int(run.info.item()) == 0, f"{tag}: info={int(run.info.item())}"
    for m, (ug, uo) in enumerate(zip(U_gpu, U_or)):
        ug = _np(ug)
        assert np.all(np.isfinite(ug)), f"{tag} mode {m}"
        eo = np.max(np.abs(ug.T @ ug - np.eye(ug.shape[1])))
        assert eo < 1e-5, f"{tag} mode {m}: U^T U - I = {eo:.2e}"
        ep = O.max_rel_err(O.projector(ug), O.projector(uo))
        assert ep <= tol, f"{tag} mode {m}: projector err {ep:.3e} > {tol}"
    return A_t, A64, U_or


def check_core_and_dw(run, lay, A_t, A64, U_or, dY_np, tol, tag, e2e_tol=None):
    U_tf = [u.astype(np.float32) for u in U_or]
    U_tf64 = [u.astype(F64) for u in U_tf]
    U_tf_t = [_dev(u) for u in U_tf]
    # core, teacher-forced factors
    S_or = O.core_project(A64, U_tf64)
    S_gpu = _np(run.core(A_t, U_tf_t))
    es = O.max_rel_err(S_gpu, S_or)
    assert es <= tol, f"{tag}: core err {es:.3e} > {tol}"
    # weight gradient, teacher-forced core and factors
    S_tf = S_or.astype(np.float32)
    dY64 = dY_np.astype(F64)
    dY_t = run.upload(dY_np)
    dW_or = _oracle_dw(lay, S_tf.astype(F64), U_tf64, dY64)
    dW_gpu = _np(run.weight_grad(dY_t, _dev(S_tf), U_tf_t))
    ew = O.max_rel_err(dW_gpu, dW_or)
    assert ew <= tol, f"{tag}: dW err {ew:.3e} > {tol}"
    # end to end with the GPU's own factors: the reconstruction S x_m U_m (Eq. 3) and dW depend on
    # the factors only through their projectors, so both are unique
    S_own = _np(run.core(A_t))
    S_ref = O.core_project(A64, U_or)
    A_hat_gpu = O.reconstruct(S_own, [_np(u) for u in run.factors()])
    A_hat_ref = O.reconstruct(S_ref, U_or)
    ea = O.max_rel_err(A_hat_gpu, A_hat_ref)
    assert ea <= tol, f"{tag}: reconstruction from the GPU's own (S, U) err {ea:.3e} > {tol}"
    del A_hat_gpu, A_hat_ref
    dW_e2e = _np(run.weight_grad(dY_t))
    dW_ref = _oracle_dw(lay, S_ref, U_or, dY64)
    ee = O.max_rel_err(dW_e2e, dW_ref)
    assert ee <= (e2e_tol or tol), f"{tag}: end-to-end dW err {ee:.3e}"
    return dW_ref


# ------------------------------------------------------------------ config 1
def test_config1_exact_tucker_full_path():
    lay = CONFIGS[1].layers[0]
    st = LayerStream(1, 0, lay)
    run = _runner(lay)
    A_np, dY_np = st.activation(0), st.grad_out(0)
    A_t, A64, U_or = check_compress(run, lay, A_np, st.u_prev0(), TOL["f32"], "cfg1")
    dW_ref = check_core_and_dw(run, lay, A_t, A64, U_or, dY_np, TOL["f32"], "cfg1")
    # exactly-Tucker activation: the compressed gradient equals the dense one (Eq. 1 on A itself)
    dense = O.conv2d_weight_grad_dense(A64, dY_np.astype(F64), _conv_spec(lay))
    assert O.max_rel_err(_np(run.dW), dense) <= TOL["f32"]
    assert O.max_rel_err(dW_ref, dense) <= 1e-5


# ------------------------------------------------------------------ configs 2 and 4: drifting sequences
def _drift_config(ci, check_at, tol):
    cfg = CONFIGS[ci]
    for li, lay in enumerate(cfg.layers):
        st = LayerStream(ci, li, lay, cfg.theta)
        run_tf, run_free = _runner(lay), _runner(lay)
        U_prev_or = [u.astype(F64) for u in st.u_prev0()]
        run_free.set_factors(st.u_prev0())
        for t in range(cfg.steps):
            tag = f"cfg{ci} layer{li} step{t}"
            A_np = st.activation(t)
            # teacher-forced: GPU starts from the oracle's previous factors (rounded to fp32)
            Uprev32 = [u.astype(np.float32) for u in U_prev_or]
            A_t, A64, U_or = check_compress(run_tf, lay, A_np, Uprev32, tol, tag)
            if t in check_at:
                check_core_and_dw(run_tf, lay, A_t, A64, U_or, st.grad_out(t), tol, tag)
            # free-running: GPU feeds on its own output
            run_free.compress(A_t)
            U_prev_or = U_or
        torch.cuda.synchronize()
        # After all steps both chains track the same subspace, to the same bar as a single step: a
        # difference between the two previous bases is contracted by (sigma_{r+1} / sigma_r)^2 per
        # step (the noise floor sits far below the weakest kept direction), so nothing accumulates.
        for m, (ug, uo) in enumerate(zip(run_free.factors(), U_prev_or)):
            ep = O.max_rel_err(O.projector(_np(ug)), O.projector(uo))
            print(f"cfg{ci} layer{li} free-running mode {m}: projector err {ep:.3e}")
            assert ep <= tol, f"cfg{ci} layer{li} free-running mode {m}: {ep:.3e}"


def test_config2_resnet18_tail_50_steps():
    _drift_config(2, check_at=(0, 1, 49), tol=TOL["f32"])


def test_config4_highres_20_steps():
    _drift_config(4, check_at=(0, 19), tol=TOL["f32"])


# ------------------------------------------------------------------ configs 3 and 5: one step, all layers
@pytest.mark.parametrize("ci", [3, 5, 6])
def test_single_step_configs(ci):
    cfg = CONFIGS[ci]
    for li, lay in enumerate(cfg.layers):
        st = LayerStream(ci, li, lay)
        run = _runner(lay)
        tol = TOL[lay.dtype]
        tag = f"cfg{ci} layer{li}"
        A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), tol, tag)
        check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), tol, tag)
        del run, A_t, A64
        torch.cuda.empty_cache()


# ------------------------------------------------------------------ edge cases
def _rand_layer(rng, dims, ranks, dtype, kind, cout, **kw):
    return Layer("edge", tuple(dims), tuple(ranks), dtype, kind, cout, alpha=0.7, noise=1e-2, **kw)


EDGE_CONV = [
    # dims, ranks, cout, k, stride, pad, dil, groups
    ((3, 5, 7, 11), (2, 3, 4, 5), 4, 3, 1, 1, 1, 1),          # ragged, nothing a multiple of a tile
    ((5, 6, 9, 8), (5, 6, 9, 8), 6, 3, 2, 0, 1, 1),            # full rank, stride 2, no padding
    ((4, 8, 10, 10), (1, 1, 1, 1), 8, 3, 1, 2, 2, 1),          # rank 1, dilation 2
    ((2, 12, 6, 5), (2, 5, 3, 2), 12, 3, 1, 1, 1, 12),         # depthwise
    ((2, 12, 6, 5), (2, 5, 3, 2), 8, 1, 1, 0, 1, 4),           # grouped pointwise
    ((1, 1, 3, 300), (1, 1, 2, 3), 2, 1, 1, 0, 1, 1),          # singleton modes, long last mode
    ((130, 3, 2, 2), (12, 3, 2, 2), 3, 2, 1, 0, 1, 1),         # long first mode, even kernel
    ((2, 70, 33, 17), (2, 20, 9, 6), 5, 5, 2, 2, 1, 1),        # 5x5 kernel, several tiles per mode
    ((3, 4, 8, 8), (2, 3, 8, 7), 5, 3, 1, 1, 1, 1),            # 8x8 planes at (almost) full rank: widest tiny-plane kernel
    ((4100, 32, 7, 7), (6, 8, 5, 5), 8, 3, 1, 1, 1, 1),        # more 7x7 planes than workgroups: each walks several tiles
    ((40, 70, 33, 31), (4, 20, 6, 5), 6, 3, 1, 1, 1, 1),       # 40920 ragged columns for the 70-channel mode: more than 32 column splits, so a tree level
    ((8, 6, 128, 128), (4, 5, 12, 12), 16, 3, 1, 1, 1, 1),       # batch of 8 over 262144 columns of grad_out: the vector-ALU product for very short modes
    ((12, 5, 150, 150), (10, 4, 9, 9), 12, 3, 1, 1, 1, 1),       # the same with 9 to 16 entries, ragged planes
    ((26, 40, 41, 45), (4, 10, 17, 9), 6, 3, 1, 1, 1, 1),        # 1040 ragged planes of three 16-blocks: the large-plane kernel, last tile partly empty
    ((17, 61, 50, 63), (3, 8, 12, 16), 5, 3, 1, 1, 1, 1),        # 1037 planes of four 16-blocks, ranks within one block
    # large maps, 3 x 3, Wo a multiple of 4: the double-buffered correlation.  37 output rows in chunks of two
    # (ragged last chunk), 70 output channels (a ragged second tile), five core channels, 50-wide slab rows
    ((2, 20, 37, 48), (2, 5, 6, 6), 70, 3, 1, 1, 1, 1),
    ((1, 9, 32, 64), (1, 4, 5, 5), 10, 3, 1, 1, 1, 1),           # 66-wide slab rows (128 lanes per row), two rows per chunk, one batch entry
    ((2, 6, 34, 32), (2, 3, 6, 5), 20, 3, 1, 1, 1, 1),           # four output rows per chunk: slabs of six rows, 34 rows in all (ragged)
    ((2, 6, 40, 68), (2, 3, 6, 5), 20, 3, 1, 2, 2, 1),           # dilation 2 over 64 output columns: six slab rows of 68 columns
    # step 5 with the sum of the partial T's in the same launch: 300 input channels (a full block of 256 and a ragged
    # one of 44), 131 output channels in pairs (the last workgroup has one), rank 40 (three K blocks, the last half empty)
    ((4, 300, 9, 9), (3, 40, 5, 5), 131, 3, 1, 1, 1, 1),
    # the same for a pointwise convolution: 1100 output channels in groups of eight (the last group has four), 130 input channels
    ((4, 130, 8, 8), (3, 24, 4, 4), 1100, 1, 1, 0, 1, 1),
    # steps 2 and 3 plane by plane in one launch: 40 x 36 planes (three 16-blocks each way, the last ones ragged),
    # ranks 12 and 8 (one K block each, partly filled); 15 planes of the core, three waves each
    ((3, 6, 40, 36), (3, 5, 12, 8), 5, 3, 1, 1, 1, 1),
    # 64 x 64 planes, ranks 32 and 20: two K blocks, the second one of the last mode a quarter full
    ((2, 5, 64, 64), (2, 3, 32, 20), 4, 3, 1, 1, 1, 1),
]


@pytest.mark.parametrize("case", EDGE_CONV)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_conv_shapes(case, dtype):
    dims, ranks, cout, k, stride, pad, dil, groups = case
    lay = Layer("edge", dims, ranks, dtype, "conv2d", cout, k=k, stride=stride, pad=pad, dil=dil,
                groups=groups, alpha=0.7, noise=1e-2)
    st = LayerStream(9, 0, lay)
    run = _runner(lay)
    tol = TOL[dtype]
    A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), tol, f"edge {case}")
    check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), tol, f"edge {case}")
    if tuple(ranks) == tuple(dims):
        # full rank: the compressed form reconstructs the activation
        S = _np(run.core(A_t))
        Ah = O.reconstruct(S, [_np(u) for u in run.factors()])
        assert O.max_rel_err(Ah, A64) <= (1e-5 if dtype == "f32" else 1e-5)


# Tensors of a million elements or more whose contiguous extent is a multiple of four take the streaming
# mode product (16-byte loads straight into the MFMA operands).  Each case names the instantiation
# <NBR, KW> it is meant to reach: NBR blocks of 16 outputs, KW waves sharing a span of 64 columns ("short": the form for modes of 17..32).  (The core
# chain starts with the mode that shrinks the tensor most, so the ranks keep H and W nearly whole.)
STREAM_CONV = [
    # a mode of 20 (two rounds, the second padded) over 144000 columns, 562.5 workgroups of 256 columns
    ((20, 16, 100, 90), (8, 8, 12, 12), 8, "short"),
    # a mode of 40 (three rounds, the last half empty) over the same columns: one wave per span in the general form
    ((40, 16, 100, 90), (8, 8, 12, 12), 16, "1, 1"),
    # 80 channels (five rounds over four waves: one wave has one round, one has none), 42000 columns = 656.25 spans
    ((5, 80, 100, 84), (4, 24, 60, 56), 12, "2, 4"),
    # 56 channels, 40 outputs (three blocks, the last half empty), two waves per span with two rounds each
    ((4, 56, 72, 76), (4, 40, 60, 68), 6, "3, 2"),
]


@pytest.mark.parametrize("case", STREAM_CONV)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_streaming_mode_product(case, dtype):
    from paper_2505_05086_amd import binding as B
    dims, ranks, cout, variant = case
    lay = Layer("stream", dims, ranks, dtype, "conv2d", cout, k=3, stride=1, pad=1, dil=1, groups=1,
                alpha=0.7, noise=1e-2)
    st = LayerStream(9, 2, lay)
    run = _runner(lay)
    tol = TOL[dtype]
    A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), tol, f"stream {case}")
    B.asi_profile_enable(True)
    try:
        check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), tol, f"stream {case}")
        sites = list(B.asi_profile_report())
    finally:
        B.asi_profile_enable(False)
    # (a bf16 tensor may take its first product along the last mode on the bf16 MFMA; the streaming product
    # then meets the fp32 intermediate)
    types = ["float"] if dtype == "f32" else ["asi::bf16_t", "float"]
    if variant == "short":          # a mode of 17..32 with one wave per span: the form without LDS
        want = ["k_ttm_stream_short<%s, 1>" % t for t in types]
    else:
        want = ["k_ttm_stream<%s, %s>" % (t, variant) for t in types]
    assert any(w in s_ for s_ in sites for w in want), (want, [s_ for s_ in sites if "ttm" in s_])


EDGE_LINEAR = [((3, 5, 7), (2, 3, 4), 6), ((4, 9, 30), (4, 9, 30), 3), ((2, 33, 130), (1, 7, 20), 70),
               ((64, 1, 5), (3, 1, 2), 1), ((6, 50, 300), (3, 34, 100), 40),     # a rank above 64
               ((3, 20, 600), (2, 8, 24), 50),                                   # a last mode of 512 or more
               # 1024 or more tokens: with bf16 data the last-mode products run on the bf16 MFMA (split factor)
               ((40, 30, 136), (5, 7, 20), 9),                                   # ragged: 1200 columns, last K chunk of 8, two output blocks
               ((36, 32, 200), (6, 8, 70), 11),                                  # five output blocks over two waves
               ((33, 32, 264), (4, 6, 100), 7),                                  # seven output blocks over four waves
               # short modes with a long inner extent (Gram-matrix route): one index (four stacked column
               # ranges), five (two ranges, a ragged second one), 20 and 40 (one and three row blocks, odd extents)
               ((1, 5, 161), (1, 3, 4), 3), ((5, 3, 700), (4, 2, 9), 5), ((20, 7, 33), (9, 3, 8), 4),
               ((40, 6, 50), (32, 4, 10), 6),
               # few tokens against a long hidden mode: the bf16 product splits its contraction over two
               # workgroups per column tile (nine chunks, the last one ragged) and sums the partial products
               ((16, 64, 520), (4, 6, 20), 8)]


@pytest.mark.parametrize("case", EDGE_LINEAR)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_linear_shapes(case, dtype):
    dims, ranks, dout = case
    lay = Layer("edge", dims, ranks, dtype, "linear", dout, alpha=0.7, noise=1e-2)
    st = LayerStream(9, 1, lay)
    run = _runner(lay)
    tol = TOL[dtype]
    A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), tol, f"edge {case}")
    check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), tol, f"edge {case}")


def test_full_rank_batch_mode_and_the_expansion_kernel_are_taken():
    """A linear layer whose batch rank equals the batch (the core is expanded along the batch mode and no G1 is
    formed) and whose last step expands rank 24 to 600 features (the vector-ALU expansion kernel: three output
    tiles, the last one ragged; 50 columns in two tiles): parity as everywhere, and the launch record shows both."""
    from paper_2505_05086_amd import binding as B
    lay = Layer("edge", (3, 20, 600), (3, 8, 24), "f32", "linear", 50, alpha=0.7, noise=1e-2)
    st = LayerStream(9, 3, lay)
    run = _runner(lay)
    A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), TOL["f32"], "expand")
    B.asi_profile_enable(True)
    try:
        check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), TOL["f32"], "expand")
        sites = list(B.asi_profile_report())
    finally:
        B.asi_profile_enable(False)
    assert any("k_ttm_expand" in s_ for s_ in sites), sites
    assert any(s_.endswith(":S1") for s_ in sites) and not any(s_.endswith(":G1") for s_ in sites), sites


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_wide_output_tiles_of_the_last_mode_pair_product(dtype):
    """P = A_m V along a last mode longer than 512 with a rank above 32 over 4096 columns: the pair product
    takes 64 outputs per workgroup (rank 40: the second block of 16 is half empty, the fourth empty; 520 rows:
    nine row tiles, the last one ragged).  Parity as everywhere, and the launch record shows the instantiation."""
    from paper_2505_05086_amd import binding as B
    lay = Layer("edge", (16, 256, 520), (4, 6, 40), dtype, "linear", 8, alpha=0.7, noise=1e-2)
    st = LayerStream(9, 5, lay)
    run = _runner(lay)
    B.asi_profile_enable(True)
    try:
        A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), TOL[dtype], "wide pair")
        sites = list(B.asi_profile_report())
    finally:
        B.asi_profile_enable(False)
    xt = "float" if dtype == "f32" else "asi::bf16_t"
    assert any("k_pair<%s, true, false, 64>" % xt in s_ for s_ in sites), sites
    check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), TOL[dtype], "wide pair")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_activation_aligned_to_its_element_only(dtype):
    """The activation may start at any element of a buffer: the tile loaders that move 16-byte pieces need an
    aligned start and have element-wise forms for the rest.  A 7 x 7 conv activation (the small-plane kernel;
    300 planes: two full tiles of 128 and a ragged third) one element into its allocation, against the oracle
    and against the same call on an aligned copy."""
    from paper_2505_05086_amd import binding as B
    lay = Layer("edge", (6, 50, 7, 7), (3, 8, 5, 5), dtype, "conv2d", 12, k=3, stride=1, pad=1, dil=1, groups=1,
                alpha=0.7, noise=1e-2)
    st = LayerStream(9, 6, lay)
    run = _runner(lay)
    A_np, U0 = st.activation(0), st.u_prev0()
    U_or = O.compress(A_np.astype(F64), [u.astype(F64) for u in U0])
    A_al = run.upload(A_np)
    buf = torch.empty(A_al.numel() + 8, dtype=A_al.dtype, device=A_al.device)
    A_off = buf[1:1 + A_al.numel()].view(A_al.shape)
    A_off.copy_(A_al)
    assert A_off.data_ptr() % 8 != 0 and A_off.is_contiguous()
    got = []
    for A_t, want in ((A_al, "true"), (A_off, "false")):
        run.set_factors(U0)
        B.asi_profile_enable(True)
        try:
            U_gpu = [_np(u).copy() for u in run.compress(A_t)]
            torch.cuda.synchronize()
            sites = list(B.asi_profile_report())
        finally:
            B.asi_profile_enable(False)
        assert int(run.info.item()) == 0
        assert any("k_subspace_tiny<" in s_ and s_.rstrip().endswith(want + ">") for s_ in sites), sites
        for m, (ug, uo) in enumerate(zip(U_gpu, U_or)):
            ep = O.max_rel_err(O.projector(ug), O.projector(uo))
            assert ep <= TOL[dtype], f"mode {m} ({want}): projector err {ep:.3e}"
        got.append(U_gpu)
    for ua, ub in zip(*got):      # the two loaders feed the same arithmetic in the same order
        assert np.array_equal(ua, ub)


def test_conv_weight_gradient_sums_the_partial_products_in_its_last_launch():
    """Ungrouped 3 x 3 and 1 x 1 convolutions: the split partial sums of the correlation (step 4 of Eq. 14) are added
    up by the launch that expands them to dW (step 5); no pass writes T out.  A 5 x 5 kernel keeps the two launches."""
    from paper_2505_05086_amd import binding as B
    for k, want_fold in ((3, True), (1, True), (5, False)):
        lay = Layer("edge", (16, 64, 14, 14), (8, 16, 7, 7), "f32", "conv2d", 64, k=k, stride=1, pad=k // 2, dil=1, groups=1,
                    alpha=0.7, noise=1e-2)
        st = LayerStream(9, 7, lay)
        run = _runner(lay)
        A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), TOL["f32"], f"fold k={k}")
        B.asi_profile_enable(True)
        try:
            check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), TOL["f32"], f"fold k={k}")
            sites = list(B.asi_profile_report())
        finally:
            B.asi_profile_enable(False)
        assert any("k_dw_fold<%d," % (k * k) in s_ for s_ in sites) == want_fold, sites
        assert any(s_.startswith("dW|k_sum_partials") for s_ in sites) == (not want_fold), sites


def test_large_planes_take_steps_2_and_3_in_one_launch():
    """Z = S x_3 U3 x_4 U4 for planes beyond 16 x 16 with ranks that are multiples of four: one launch, a wave per plane
    of the core (48 x 52 planes, ranks 16 and 24); with a rank that is not a multiple of four, the two mode products."""
    from paper_2505_05086_amd import binding as B
    for ranks, fused in (((3, 4, 16, 24), True), ((3, 4, 16, 22), False)):
        lay = Layer("edge", (4, 6, 48, 52), ranks, "f32", "conv2d", 7, k=3, stride=1, pad=1, dil=1, groups=1, alpha=0.7, noise=1e-2)
        st = LayerStream(9, 8, lay)
        run = _runner(lay)
        A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), TOL["f32"], f"z planes {ranks}")
        B.asi_profile_enable(True)
        try:
            check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), TOL["f32"], f"z planes {ranks}")
            sites = list(B.asi_profile_report())
        finally:
            B.asi_profile_enable(False)
        assert any("k_z_planes<4>" in s_ for s_ in sites) == fused, sites
        assert any(s_.endswith(":Z1") for s_ in sites) == (not fused), sites


def test_core_projection_takes_the_two_plane_modes_in_one_launch():
    """The H and W products of the core projection on an fp32 intermediate with 48 x 52 planes (three and four
    16-blocks, both ragged; ranks 16 and 24): one launch, a workgroup per plane, after the channel mode has shrunk the
    tensor; the core, the reconstruction and the weight gradient are checked like anywhere else."""
    from paper_2505_05086_amd import binding as B
    lay = Layer("edge", (4, 24, 48, 52), (3, 6, 16, 24), "f32", "conv2d", 7, k=3, stride=1, pad=1, dil=1, groups=1, alpha=0.7, noise=1e-2)
    st = LayerStream(9, 9, lay)
    run = _runner(lay)
    A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), TOL["f32"], "core planes")
    B.asi_profile_enable(True)
    try:
        check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), TOL["f32"], "core planes")
        sites = list(B.asi_profile_report())
    finally:
        B.asi_profile_enable(False)
    assert any("k_core_planes<4>" in s_ for s_ in sites), sites


def test_rank_above_192_takes_the_general_orthogonalisation():
    """Ranks in (192, 1024] leave the blocked orthogonalisation kernels for the single-workgroup one and
    need 13 or more rank tiles in the product kernels; the whole path is checked like any other shape."""
    lay = Layer("edge", (8, 40, 600), (8, 40, 200), "f32", "linear", 9, alpha=0.3, noise=1e-2)
    st = LayerStream(9, 4, lay)
    run = _runner(lay)
    A_t, A64, U_or = check_compress(run, lay, st.activation(0), st.u_prev0(), TOL["f32"], "rank 200")
    check_core_and_dw(run, lay, A_t, A64, U_or, st.grad_out(0), TOL["f32"], "rank 200")


def test_accumulate_adds_to_dw_and_aliasing_factors_is_allowed():
    import paper_2505_05086_amd as asi
    lay = Layer("edge", (4, 6, 5, 5), (2, 3, 2, 2), "f32", "conv2d", 6, k=3, pad=1, alpha=0.5, noise=1e-2)
    st = LayerStream(9, 2, lay)
    run = _runner(lay)
    A_t = run.upload(st.activation(0))
    dY_t = run.upload(st.grad_out(0))
    run.set_factors(st.u_prev0())
    run.compress(A_t)
    U_sep = [u.clone() for u in run.factors()]
    # same call with U_out aliasing U_prev
    alias = [_dev(u) for u in st.u_prev0()]
    asi.asi_compress(run.desc, A_t, alias, alias, run.ws, run.info)
    torch.cuda.synchronize()
    for a, b in zip(alias, U_sep):
        assert torch.equal(a, b)
    run.core(A_t)
    once = run.weight_grad(dY_t).clone()
    twice = run.weight_grad(dY_t, accumulate=True).clone()
    assert torch.allclose(twice, 2 * once, rtol=1e-6, atol=1e-6)


def test_runs_are_bitwise_reproducible():
    lay = CONFIGS[2].layers[1]
    st = LayerStream(2, 1, lay)
    A_np, dY_np = st.activation(0), st.grad_out(0)
    outs = []
    for _ in range(2):
        run = _runner(lay)
        run.set_factors(st.u_prev0())
        dW = run.step(run.upload(A_np), run.upload(dY_np))
        torch.cuda.synchronize()
        outs.append([dW.clone(), run.S.clone()] + [u.clone() for u in run.factors()])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_rank_deficient_input_sets_info():
    lay = Layer("edge", (4, 6, 5, 5), (2, 3, 2, 2), "f32", "conv2d", 6, k=3, pad=1)
    run = _runner(lay)
    run.set_factors(LayerStream(9, 3, lay).u_prev0())
    run.compress(torch.zeros(lay.dims, device="cuda"))
    torch.cuda.synchronize()
    code = int(run.info.item())
    assert code != 0 and 1 <= code // 1000 <= 4 and 1 <= code % 1000 <= 3
    # the oracle refuses the same input
    with pytest.raises(O.OrthogonalizeBreakdown):
        O.compress(np.zeros(lay.dims), [np.eye(n)[:, :r] for n, r in zip(lay.dims, lay.ranks)])
    # a following good call clears it
    st = LayerStream(9, 3, lay)
    run.set_factors(st.u_prev0())          # the failed call left unspecified factors behind
    run.compress(run.upload(st.activation(0)))
    torch.cuda.synchronize()
    assert int(run.info.item()) == 0


def _graded_tensor(lay, ratio, seed=20250505):
    """Tucker tensor whose factor columns decay geometrically to `ratio`: an ill-conditioned P."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal(lay.ranks)
    for m, (n, r) in enumerate(zip(lay.dims, lay.ranks)):
        q, _ = np.linalg.qr(rng.standard_normal((n, r)))
        q = q * (ratio ** (np.arange(r) / (r - 1)))[None, :]       # column j scaled by ratio^(j/(r-1))
        A = np.moveaxis(np.tensordot(q, A, axes=(1, m)), 0, m)
    return (A / np.max(np.abs(A))).astype(np.float32)


def _check_orthonormal_basis(lay, A, stream_id, tag):
    st = LayerStream(9, stream_id, lay)
    run = _runner(lay)
    run.set_factors(st.u_prev0())
    U_gpu = run.compress(run.upload(A))
    torch.cuda.synchronize()
    assert int(run.info.item()) == 0, tag
    A64 = A.astype(F64)
    U0 = [u.astype(F64) for u in st.u_prev0()]
    U_or = O.compress(A64, U0)
    eps32 = 2.0 ** -24
    compared = 0
    for m, (ug, uo) in enumerate(zip(U_gpu, U_or)):
        ug = _np(ug)
        assert np.all(np.isfinite(ug))
        r = ug.shape[1]
        eo = np.max(np.abs(ug.T @ ug - np.eye(r)))
        assert eo < 1e-5, f"{tag} mode {m}: U^T U - I = {eo:.2e}"
        # Gram-Schmidt keeps the column order of P, so the first k columns of the factor span the
        # first k columns of P on both sides.  The library rounds V = A_m^T U_prev to fp32 (the fp32
        # path's own arithmetic), which perturbs P by about eps32 ||A_m||^2 ||U_prev|| sqrt(b_m) at worst, and the span of
        # P[:, :k] moves by that over sigma_min(P[:, :k]).  Each nested projector is therefore held to
        #     8 eps32 sigma_max(P) / sigma_min(P[:, :k])    (plus the 1e-6 floor of the fp32 output),
        # with the conditioning taken from the oracle's P; leading blocks whose bound exceeds 0.1 are
        # not comparable in fp32 and are skipped.
        Pm = O.subspace_P(A64, U0[m], m)
        smax = np.linalg.svd(Pm, compute_uv=False)[0]
        for k in range(1, r + 1):
            smin_k = np.linalg.svd(Pm[:, :k], compute_uv=False)[-1]
            bound = 8.0 * eps32 * smax / smin_k + 1e-6
            if bound > 0.1:
                break
            ep = np.max(np.abs(O.projector(ug[:, :k]) - O.projector(uo[:, :k])))
            assert ep <= bound, f"{tag} mode {m}: leading {k} columns, projector err {ep:.2e} > bound {bound:.2e}"
            compared += 1
    assert compared >= len(U_or), f"{tag}: only {compared} nested projectors were comparable"


@pytest.mark.parametrize("ratio", [1e-1, 1e-2, 3e-3])
def test_ill_conditioned_subspace_product_stays_orthonormal(ratio):
    """cond(P), P = A_m (A_m^T U), grows like ratio^-3 here: ~1e3 at 0.1 (settled by the first
    Cholesky-QR pass), up to 1e6 at 0.01 (needs the second pass), 5e7 at 0.003 (mode 2 loses a
    pivot to the 1e-12 threshold in the plain factorisation and takes the shifted one).
    The basis must come out orthonormal to fp32 rounding on every route, and must
    contain the dominant directions the oracle finds (the weakest ones are below the fp32 rounding
    of V and are not comparable)."""
    lay = Layer("illcond", (16, 40, 9, 9), (6, 12, 4, 4), "f32", "conv2d", 8, k=3, pad=1)
    _check_orthonormal_basis(lay, _graded_tensor(lay, ratio), 7, f"ratio {ratio}")


@pytest.mark.parametrize("ratio", [0.3, 0.05])
def test_ill_conditioned_wide_rank_stays_orthonormal(ratio):
    """The same for a rank above 64 (the wide orthogonalisation kernels): for the 90-column mode
    cond(P) is 4e5 at 0.3 (second pass needed) and 5e8 at 0.05 (a pivot falls below 1e-12 of its
    diagonal entry: shifted retry).  The well-conditioned route of these kernels (second pass
    skipped) is covered by the rank-100 case of the linear edge shapes."""
    lay = Layer("illcond", (8, 40, 260), (6, 16, 90), "f32", "linear", 12)
    _check_orthonormal_basis(lay, _graded_tensor(lay, ratio), 8, f"wide ratio {ratio}")


@pytest.mark.parametrize("ratio", [0.3, 0.05])
def test_ill_conditioned_wide_rank_many_slices(ratio):
    """A wide mode long enough (2100 rows: 17 slices of 128) that its slice Gram matrices are added
    by a tree level before the factorisation; both passes and the shifted retry read the summed ones."""
    lay = Layer("illcond", (8, 20, 2100), (6, 16, 90), "f32", "linear", 12)
    _check_orthonormal_basis(lay, _graded_tensor(lay, ratio), 10, f"wide, many slices, ratio {ratio}")
