"""Host-side checks of the synthetic input recipe (no method arithmetic involved)."""
import numpy as np

from asi_inputs import CONFIGS, LayerStream, bf16_bits_to_f32, f32_to_bf16_bits
from asi_inputs.synth import cayley_rotation, round_to_dtype


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -2.5, 0.0, 3.3895313892515355e38],
                 dtype=np.float32)
    b = bf16_bits_to_f32(f32_to_bf16_bits(x))
    assert b[0] == 1.0 and b[1] == 1.0            # tie -> even mantissa
    assert b[2] == np.float32(1.0 + 2 ** -6)      # tie -> even (up)
    assert b[3] == np.float32(1.0 + 2 ** -7)
    assert b[4] == -2.5 and b[5] == 0.0
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    rb = bf16_bits_to_f32(f32_to_bf16_bits(r))
    assert np.max(np.abs(rb - r) / np.abs(r)) <= 2.0 ** -8
    assert np.array_equal(bf16_bits_to_f32(f32_to_bf16_bits(rb)), rb)


def test_cayley_is_orthogonal_small_angle():
    rng = np.random.default_rng(1)
    R = cayley_rotation(rng, 20, 0.02)
    assert np.max(np.abs(R.T @ R - np.eye(20))) < 1e-13
    ang = np.max(np.abs(np.angle(np.linalg.eigvals(R))))
    assert 0.015 < ang < 0.0201


def test_config1_is_exact_tucker_plus_tiny_noise():
    lay = CONFIGS[1].layers[0]
    st = LayerStream(1, 0, lay)
    A = st.activation(0).astype(np.float64)
    assert A.shape == lay.dims and abs(np.sqrt(np.mean(A * A)) - 1.0) < 1e-3
    for m, r in enumerate(lay.ranks):
        s = np.linalg.svd(np.moveaxis(A, m, 0).reshape(A.shape[m], -1), compute_uv=False)
        assert s[r] / s[r - 1] < 1e-3             # rank r up to noise + float32 rounding


def test_config2_spectrum_decays_and_drifts_slowly():
    lay = CONFIGS[2].layers[1]
    st = LayerStream(2, 1, lay)
    A0 = st.activation(0).astype(np.float64)
    s = np.linalg.svd(np.moveaxis(A0, 1, 0).reshape(512, -1), compute_uv=False)
    assert s[0] ** 2 / np.sum(s ** 2) > 0.5       # first singular value carries most energy
    assert s[47] / s[48] > 5                      # signal sits well above the noise floor
    f0, f1 = st.true_factors(0), st.true_factors(1)
    for a, b in zip(f0, f1):
        sv = np.linalg.svd(a.T @ b, compute_uv=False)
        assert 0.9995 < sv.min() <= 1.0 + 1e-12 and sv.min() < 1.0 - 1e-8
    # restarting the stream reproduces the same tensors
    st2 = LayerStream(2, 1, lay)
    assert np.array_equal(st2.activation(1), st.activation(1))
    assert np.array_equal(st2.grad_out(3), st.grad_out(3))
    assert st.grad_out(0).shape == (64, 512, 7, 7)


def test_u_prev0_orthonormal_and_layer_shapes():
    for ci, cfg in CONFIGS.items():
        for li, lay in enumerate(cfg.layers):
            assert len(lay.dims) == len(lay.ranks)
            assert all(1 <= r <= n for r, n in zip(lay.ranks, lay.dims))
    st = LayerStream(3, 0, CONFIGS[3].layers[0])
    for u in st.u_prev0():
        assert u.dtype == np.float32
        assert np.max(np.abs(u.T.astype(np.float64) @ u - np.eye(u.shape[1]))) < 1e-6
    assert CONFIGS[3].layers[1].dw_shape == (960, 1, 3, 3)
    assert CONFIGS[5].layers[1].grad_out_shape == (64, 197, 768)
    assert round_to_dtype(np.array([1.0 + 2 ** -10]), "bf16")[0] == 1.0
