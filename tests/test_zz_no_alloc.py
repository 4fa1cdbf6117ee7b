"""plora_delta_static (the entry point for callers that cannot allocate: v lives in the library's static
device array) against plora_delta with caller-owned v buffers, through the C ABI: two calls in a row on
one pool, the second with a smaller batch and fewer slots, each compared bit for bit with the existing
entry point (same kernels, same order of sums) and, within the stated tolerances, with the oracle; plus
the size limit."""
import numpy as np
import pytest

from workload import DT_BF16, Layout, draw_tok2adapter, from_elt, make_act
from helpers import TOL_Y, Case, raw_to_torch, rel_err, torch_to_raw

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_plora_delta(oracle_mod):
    import torch
    import paper_2512_20210_amd as P
    lay = Layout((1024, 520, 256, 1024), (1024, 264, 1544, 512), DT_BF16)
    ranks = [8, 16, 3, 40, 64, 24, 32, 5]
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], 16384, 512, seed=43)
    pool = case.gpool
    rng = np.random.default_rng(5)
    for T, slots, mfma in ((300, [0, 1, 2, 3], 2), (37, [1, 2], 0)):   # the second call is the smaller one
        case.set_mfma(mfma)
        t2a = draw_tok2adapter(rng, T, np.arange(len(ranks)), s=1.0, none_frac=0.1)
        xs = [make_act(rng, T, lay.d_in[s], lay.dtype) for s in slots]
        y0 = [make_act(rng, T, lay.d_out[s], lay.dtype) for s in slots]
        xd = [raw_to_torch(a, "cuda") for a in xs]
        y_a = [raw_to_torch(a, "cuda") for a in y0]
        y_b = [raw_to_torch(a, "cuda") for a in y0]
        vd = [torch.full((T, case.max_rank), float("nan"), device="cuda") for _ in slots]
        batch = pool.batch_begin(t2a, case.stream)
        print("no-alloc: T=%d slots=%s mfma_min_tokens=%d" % (T, slots, mfma), flush=True)
        pool.delta(batch, slots[0], xd, vd, y_a, case.stream)
        pool.delta_static(batch, slots[0], xd, y_b, case.stream)
        pool.batch_end(batch)
        torch.cuda.synchronize()
        for q, s in enumerate(slots):
            assert torch.equal(y_a[q], y_b[q]), "slot %d: static workspace gives another y than caller-owned v" % s
            v_ref = case.opool.shrink(s, xs[q], t2a, acc64=True)
            y_ref = case.opool.expand(s, v_ref, t2a, y0[q].copy(), acc64=True)
            err = rel_err(from_elt(torch_to_raw(y_b[q], lay.dtype), lay.dtype), from_elt(y_ref, lay.dtype))
            assert err <= TOL_Y[lay.dtype], "slot %d: y error %.3g" % (s, err)
    # beyond the array's 16 MiB: refused, nothing queued (4 slots x 20000 tokens x 64 floats = 20.5 MB)
    T = 20000
    t2a = np.zeros(T, np.int32)
    batch = pool.batch_begin(t2a, case.stream)
    dummy = torch.zeros(8, dtype=torch.int16, device="cuda")
    rc = P.plora_delta_static(pool.h, batch, 0, 4, [dummy.data_ptr()] * 4, [dummy.data_ptr()] * 4, case.stream)
    assert rc == P.PLORA_ERR_LIMIT
    pool.batch_end(batch)
    case.close()
