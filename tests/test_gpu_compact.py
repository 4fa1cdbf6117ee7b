"""GPU tests of plora_compact (Sec. III-C "Defragmentation"): pages moved on the device while batches
that read them are still in flight, loads into the vacated pages right behind, everything compared
with the oracle (page tables, slab bytes through the tables, batch results)."""
import numpy as np
import pytest

from workload import DT_BF16, DT_F16, Layout, from_elt, to_elt
from helpers import Case, TOL_V, TOL_Y, raw_to_torch, rel_err, torch_to_raw

pytestmark = pytest.mark.gpu


def _tables_equal(case, ids):
    for i in ids:
        assert case.gpool.page_table(i).tolist() == case.opool.page_table(i).tolist(), "page table of adapter %d" % i


def _slab_holds_blobs(case, slab, ids, page_bytes):
    pages = slab.view(-1, page_bytes).cpu().numpy()
    for i in ids:
        raw = case.blobs[i].view(np.uint8).reshape(-1)
        got = pages[case.opool.page_table(i)].reshape(-1)[:len(raw)]
        assert (got == raw).all(), "slab bytes of adapter %d differ from its blob" % i


@pytest.mark.parametrize("dtype,page_bytes", [(DT_BF16, 4096), (DT_F16, 16384)])
def test_compaction_under_batches_in_flight(oracle_mod, dtype, page_bytes):
    import torch
    lay = Layout((520, 256), (264, 1024), dtype)
    C = sum(lay.d_in) + sum(lay.d_out)
    ranks = [8, 16, 40, 64, 5, 33, 12, 64, 24, 3, 48, 16]
    pages_of = lambda r: -(-(r * 2 * C) // page_bytes)
    n_pages = sum(pages_of(r) for r in ranks) + 6
    slab = torch.zeros(n_pages * page_bytes, dtype=torch.uint8, device="cuda")
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], page_bytes, n_pages, seed=71,
                load_order=list(range(8)), mfma_min_tokens=6, slab=slab)
    g, o = case.gpool, case.opool
    rng = np.random.default_rng(72)
    # evict every other adapter, load others over and behind the holes (they end up scattered), then open
    # new holes below
    for i in (0, 2, 4, 6):
        case.evict(i)
    for i in (8, 9, 10):
        case.load(i)
    for i in (1, 3):
        case.evict(i)
    resident = [5, 7, 8, 9, 10]
    scattered = sum(np.any(np.diff(o.page_table(i)) != 1) for i in resident)
    assert scattered >= 2, "the history was meant to scatter some adapters"
    torch.cuda.synchronize()

    # a batch whose kernels are queued but not waited for, then the compaction on the copy stream, a load
    # into the vacated pages on the compute stream, and a second batch over moved and new adapters
    T = 96
    t2a_1 = np.asarray(rng.choice(resident, size=T), np.int32)
    x_raw = [to_elt(rng.standard_normal((T, d)).astype(np.float32), dtype) for d in lay.d_in]
    y0_raw = [to_elt(rng.standard_normal((T, d)).astype(np.float32), dtype) for d in lay.d_out]
    xd = [raw_to_torch(x, "cuda") for x in x_raw]
    stream = torch.cuda.current_stream().cuda_stream

    def queue_batch(t2a):
        yd = [raw_to_torch(y, "cuda") for y in y0_raw]
        vd = [torch.full((T, case.max_rank), float("nan"), device="cuda", dtype=torch.float32) for _ in lay.d_in]
        b = g.batch_begin(t2a, stream)
        g.shrink(b, 0, xd, vd, stream)
        g.expand(b, 0, vd, yd, stream)
        g.batch_end(b)
        return vd, yd

    def reference(t2a):
        out = []
        for s in range(lay.n_slots):
            v = o.shrink(s, x_raw[s], t2a, acc64=True)
            out.append((v, o.expand(s, v, t2a, y0_raw[s].copy(), acc64=True)))
        return out

    ref_1 = reference(t2a_1)  # with the tables as they are now
    queued_1 = queue_batch(t2a_1)
    before = {i: o.page_table(i).tolist() for i in resident}
    got = g.compact(case.copy_stream.cuda_stream)
    want = o.compact()
    assert got == want and got[1] >= 2, (got, want)
    _tables_equal(case, resident)
    moved = [i for i in resident if o.page_table(i).tolist() != before[i]]
    print("compaction moved", got, "adapters", moved, flush=True)
    assert g.stats()["compacted_pages"] == got[0]
    # right behind it, loads that land in the vacated pages (other stream than the moves)
    for i in (11, 0):
        pt_o = o.load(i, ranks[i], case.scales[i], case.blobs[i])
        pt_g = g.load(i, ranks[i], case.scales[i], case.pinned[i], stream)
        assert pt_g.tolist() == pt_o.tolist()
    resident += [11, 0]
    t2a_2 = np.asarray(rng.choice(moved + [11, 0], size=T), np.int32)
    ref_2 = reference(t2a_2)
    queued_2 = queue_batch(t2a_2)
    torch.cuda.synchronize()
    for (vd, yd), ref in ((queued_1, ref_1), (queued_2, ref_2)):
        for s in range(lay.n_slots):
            v_ref, y_ref = ref[s]
            assert rel_err(vd[s].cpu().numpy(), v_ref) <= TOL_V
            assert rel_err(from_elt(torch_to_raw(yd[s], dtype), dtype), from_elt(y_ref, dtype)) <= TOL_Y[dtype]
    _slab_holds_blobs(case, slab, resident, page_bytes)
    st = g.stats()
    assert st["compacted_adapters"] == got[1] and st["compact_ms"] > 0.0

    # a second call finds nothing to do; with a bound the moves come in steps, each as the oracle's
    assert g.compact(case.copy_stream.cuda_stream) == (0, 0) and o.compact() == (0, 0)
    for i in (5, 7, 9):
        case.evict(i)
        resident.remove(i)
    steps = 0
    while True:
        got, want = g.compact(case.copy_stream.cuda_stream, max_pages=6), o.compact(max_pages=6)
        assert got == want
        _tables_equal(case, resident)
        torch.cuda.synchronize()  # (an adapter whose move is in flight would sit the next step out)
        steps += 1
        if got == (0, 0) or steps > 50:
            break
    torch.cuda.synchronize()
    _slab_holds_blobs(case, slab, resident, page_bytes)
    # the usual parity run over everything that is resident now (all kernel modes)
    case.run(np.asarray(rng.choice(resident, size=64), np.int32), seed=5)
    case.close()
