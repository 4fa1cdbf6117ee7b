"""plora_shrink / plora_expand under HIP graph capture: they enqueue kernels only (no allocation, no
memset, no event when profiling is off), so a step over an open batch can be captured once and
replayed.  Every replay is checked against the oracle and, bit for bit, against the eager result,
with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from workload import DT_BF16, Layout, draw_tok2adapter, from_elt, make_act
from helpers import TOL_V, TOL_Y, Case, raw_to_torch, rel_err, torch_to_raw

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mfma", [0, 2])
def test_captured_step_replays_to_the_eager_result(oracle_mod, mfma):
    import torch
    lay = Layout((1024, 520), (1024, 264), DT_BF16)
    ranks = [8, 16, 3, 40, 64, 24, 32, 5]
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], 16384, 256, seed=41, mfma_min_tokens=mfma)
    pool = case.gpool
    rng = np.random.default_rng(3)
    T = 150
    t2a = draw_tok2adapter(rng, T, np.arange(len(ranks)), s=1.0, none_frac=0.1)
    xs = [make_act(rng, T, d, lay.dtype) for d in lay.d_in]
    y0 = [make_act(rng, T, d, lay.dtype) for d in lay.d_out]
    xd = [raw_to_torch(a, "cuda") for a in xs]
    y_init = [raw_to_torch(a, "cuda") for a in y0]
    yd = [t.clone() for t in y_init]
    vd = [torch.full((T, case.max_rank), float("nan"), device="cuda") for _ in xs]
    side = torch.cuda.Stream()
    batch = pool.batch_begin(t2a, side.cuda_stream)   # the image copy and its event stay outside the graph
    # eager
    pool.shrink(batch, 0, xd, vd, side.cuda_stream)
    pool.expand(batch, 0, vd, yd, side.cuda_stream)
    torch.cuda.synchronize()
    v_eager = [t.clone() for t in vd]
    y_eager = [t.clone() for t in yd]
    for s in range(lay.n_slots):
        v_ref = case.opool.shrink(s, xs[s], t2a, acc64=True)
        y_ref = case.opool.expand(s, v_ref, t2a, y0[s].copy(), acc64=True)
        assert rel_err(v_eager[s].cpu().numpy(), v_ref) <= TOL_V
        assert rel_err(from_elt(torch_to_raw(y_eager[s], lay.dtype), lay.dtype), from_elt(y_ref, lay.dtype)) <= TOL_Y[lay.dtype]
    # capture the same two calls
    for t, src in zip(yd, y_init):
        t.copy_(src)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        pool.shrink(batch, 0, xd, vd, side.cuda_stream)
        pool.expand(batch, 0, vd, yd, side.cuda_stream)
    for replay in range(4):
        for t, src in zip(yd, y_init):   # eager work between the replays
            t.copy_(src)
        for t in vd:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for s in range(lay.n_slots):
            assert torch.equal(vd[s], v_eager[s]), "replay %d, slot %d: v differs from the eager run" % (replay, s)
            assert torch.equal(yd[s], y_eager[s]), "replay %d, slot %d: y differs from the eager run" % (replay, s)
    pool.batch_end(batch)
    case.close()
