"""A captured HIP graph of one layer-step must reproduce the eager result on every replay,
also with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from asi_inputs import CONFIGS, LayerStream

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    from paper_2505_05086_amd.runner import LayerRunner
    lay = CONFIGS[2].layers[1]
    st = LayerStream(2, 1, lay)
    A_np = [st.activation(t) for t in range(3)]
    dY_np = [st.grad_out(t) for t in range(3)]

    def fresh():
        r = LayerRunner(lay)
        r.set_factors(st.u_prev0())
        return r

    # eager reference: three consecutive steps
    ref = fresh()
    A = [ref.upload(a) for a in A_np]
    dY = [ref.upload(g) for g in dY_np]
    eager = []
    for t in range(3):
        dW = ref.step(A[t], dY[t])
        torch.cuda.synchronize()
        eager.append((dW.clone(), ref.S.clone(), [u.clone() for u in ref.factors()]))

    # the same three steps, each from a captured graph (static input buffers, refilled before a replay)
    run = fresh()
    A_in, dY_in = torch.empty_like(A[0]), torch.empty_like(dY[0])
    A_in.copy_(A[0]); dY_in.copy_(dY[0])
    side = torch.cuda.Stream()
    graphs = []
    with torch.cuda.stream(side):
        run.step(A_in, dY_in); run.step(A_in, dY_in)          # warm-up outside capture (even count)
        torch.cuda.synchronize()
        for _ in range(2):                                   # two graphs: the factor buffers alternate
            g = torch.cuda.CUDAGraph()
            g.capture_begin()
            run.step(A_in, dY_in)
            g.capture_end()
            graphs.append(g)
    torch.cuda.synchronize()
    for rep in range(3):                                     # several rounds of replays
        run.cur = 0
        run.set_factors(st.u_prev0())
        for t in range(3):
            A_in.copy_(A[t]); dY_in.copy_(dY[t])
            junk = (A_in * 2).sum()                          # unrelated eager work between replays
            torch.cuda.synchronize()
            graphs[t % 2].replay()
            torch.cuda.synchronize()
            run.cur = 1 - run.cur                            # the replay flipped the buffers on the device side
            dW_e, S_e, U_e = eager[t]
            assert torch.equal(run.dW, dW_e), f"replay round {rep} step {t}: dW differs"
            assert torch.equal(run.S, S_e)
            for a, b in zip(run.factors(), U_e):
                assert torch.equal(a, b)
            assert int(run.info.item()) == 0 and float(junk) == float(junk)
