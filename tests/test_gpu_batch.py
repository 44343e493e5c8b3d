"""Batched entry points: every launch serves several layers.  The factors must be bit-identical to
the single-layer calls (which the parity tests check against the float64 oracle); core and weight
gradient may differ at fp32 rounding level, because a batch takes the m-mode products of the
core projection in one common order."""
import numpy as np
import pytest
import torch

from asi_inputs import CONFIGS, LayerStream
from paper_2505_05086_amd.runner import BatchRunner, LayerRunner

pytestmark = pytest.mark.gpu


def _run_pair(cfg_index, layer_ids, steps=2):
    cfg = CONFIGS[cfg_index]
    layers = [cfg.layers[i] for i in layer_ids]
    streams = [LayerStream(cfg.index, i, cfg.layers[i], cfg.theta) for i in layer_ids]
    singles = [LayerRunner(lay) for lay in layers]
    batch = BatchRunner(layers)
    for r, b, st in zip(singles, batch.runs, streams):
        r.set_factors(st.u_prev0())
        b.set_factors(st.u_prev0())
    for t in range(steps):
        A = [r.upload(st.activation(t)) for r, st in zip(singles, streams)]
        dY = [r.upload(st.grad_out(t)) for r, st in zip(singles, streams)]
        for r, a, g in zip(singles, A, dY):
            r.step(a, g)
        batch.step(A, dY)
        torch.cuda.synchronize()
        for li, (r, b) in enumerate(zip(singles, batch.runs)):
            assert int(r.info.item()) == 0 and int(b.info.item()) == 0
            for m, (u1, u2) in enumerate(zip(r.factors(), b.factors())):
                assert torch.equal(u1, u2), f"cfg{cfg_index} layer {layer_ids[li]} step {t} factor {m}"
            for name, x, y in (("core", r.S, b.S), ("dW", r.dW, b.dW)):
                err = float((x - y).abs().max() / x.abs().max())
                assert err <= 2e-6, f"cfg{cfg_index} layer {layer_ids[li]} step {t} {name}: {err:.2e}"


def test_batch_equals_single_config2_all_layers():
    _run_pair(2, [0, 1, 2, 3])


def test_batch_equals_single_config3_mixed_shapes_and_groups():
    _run_pair(3, list(range(len(CONFIGS[3].layers))))


def test_batch_equals_single_config5_linear_bf16():
    _run_pair(5, list(range(len(CONFIGS[5].layers))), steps=1)


def test_batch_of_one_and_repeated_layer():
    _run_pair(1, [0])
    _run_pair(2, [1, 1, 2])


def test_batch_of_eight_layers():
    """The largest batch the ABI takes: every launch serves eight argument blocks."""
    _run_pair(2, [0, 1, 2, 3, 3, 2, 1, 0], steps=1)
    _run_pair(3, [0, 3, 0, 3, 1, 2, 0, 3], steps=1)
