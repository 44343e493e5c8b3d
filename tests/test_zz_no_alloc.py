"""The entry point that allocates nothing (asi_compress_static: the library's static device
array in place of a caller workspace) against asi_compress on the same inputs, through the
C ABI: two calls in a row, the second on a smaller layer, so that what the first call left in
the shared array must not matter.  The two entry points run the same kernels, so the factors
must agree bit for bit (the parity bar of the fp32 path, 1e-4 on projectors, is implied)."""
import gc

import numpy as np
import pytest
import torch

import paper_2505_05086_amd as asi
from asi_inputs import CONFIGS, LayerStream
from asi_inputs.configs import Layer
from oracle import asi_oracle as O

pytestmark = pytest.mark.gpu


def _compress_both(lay, stream_id):
    from paper_2505_05086_amd.runner import LayerRunner
    st = LayerStream(9, stream_id, lay)
    run = LayerRunner(lay)
    A_np, U0 = st.activation(0), st.u_prev0()
    A_t = run.upload(A_np)
    run.set_factors(U0)
    ref = [u.clone() for u in run.compress(A_t)]              # existing entry point, caller workspace
    torch.cuda.synchronize()
    assert int(run.info.item()) == 0
    prev = [torch.from_numpy(np.ascontiguousarray(u, dtype=np.float32)).cuda() for u in U0]
    out = [torch.full_like(u, float("nan")) for u in ref]
    info = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    # no allocation through torch's allocator during the call: the cumulative count of allocations stands still
    # (the bytes in use may drop meanwhile, when Python collects what earlier tests left behind)
    gc.collect()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    asi.asi_compress_static(run.desc, A_t, prev, out, info)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    assert int(info.item()) == 0
    for m, (a, b) in enumerate(zip(out, ref)):
        assert torch.equal(a, b), f"mode {m}: static-scratch result differs from the workspace result"
    U_or = O.compress(A_np.astype(np.float64), [u.astype(np.float64) for u in U0])
    for m, (a, uo) in enumerate(zip(out, U_or)):
        ep = O.max_rel_err(O.projector(a.cpu().numpy().astype(np.float64)), O.projector(uo))
        assert ep <= 1e-4, f"mode {m}: projector error {ep:.2e} against the oracle"


def test_static_scratch_two_calls_second_smaller():
    big = CONFIGS[2].layers[0]                                # (64,256,14,14): ~10 MB of scratch, every kernel family
    small = Layer("edge", (5, 70, 9, 11), (3, 20, 4, 5), "f32", "conv2d", 4, k=3, pad=1, alpha=0.7, noise=1e-2)
    _compress_both(big, 20)
    _compress_both(small, 21)
    _compress_both(big, 22)                                   # and a larger one again after the small one


def test_static_scratch_rejects_layers_beyond_its_size():
    lay = CONFIGS[5].layers[1]
    d = asi.make_desc(lay.dims, lay.ranks, lay.dtype)
    assert asi.asi_workspace_bytes(d) > asi.binding.STATIC_SCRATCH_BYTES
    x = torch.zeros(1, device="cuda")
    with pytest.raises(asi.AsiError) as e:
        asi.asi_compress_static(d, x, [x] * 3, [x] * 3, None)
    assert e.value.status == 3
