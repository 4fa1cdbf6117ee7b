"""Full-size workloads in the launch configuration bench.py times, checked on sampled outputs.

The oracle cannot run a whole step at these sizes in seconds, so it recomputes sampled
(slot, token) rows one by one (fp64 accumulation) through its own page pool holding the same
adapters; page tables and the batch translation are compared in full, and the properties that hold
at any size (v is zero beyond each token's rank, untouched rows stay untouched) are checked on
every slot.
"""
import time

import numpy as np
import pytest

from workload import from_elt
from helpers import TOL_V, TOL_Y, rel_err, torch_to_raw

pytestmark = pytest.mark.gpu


def _run(oracle_mod, name, n_slots_checked, n_tok_checked):
    import torch
    import bench
    t0 = time.time()
    w = bench.GpuWorkload(name, verbose=True)
    lay, cfg = w.lay, w.cfg
    rng = np.random.default_rng(cfg["seed"] + 7)
    t2a = bench.draw_batch(cfg, rng, w.n_ad)
    T = len(t2a)
    w.alloc_activations(T, cfg["seed"] + 9)
    print("%s: built in %.1fs, T=%d" % (name, time.time() - t0, T), flush=True)
    # poison v so that unwritten entries show
    for v in w.v:
        v.fill_(float("nan"))
    w.step(t2a, lay.n_slots)  # one call over all slots, as bench.py does by default
    torch.cuda.synchronize()
    print("%s: step done" % name, flush=True)

    # oracle pool with the same adapters, same order
    op = oracle_mod.OraclePool(w.page_bytes, w.n_pages, lay.d_in, lay.d_out, lay.dtype, w.n_ad, w.max_rank)
    for i in range(w.n_ad):
        pt = op.load(i, int(w.ranks[i]), w.scales[i], w.blobs[i])
        assert pt.tolist() == w.tables[i].tolist(), "page table of adapter %d differs" % i
    b = w.pool.batch_begin(t2a, w.stream)
    perm, sa, ss = w.pool.batch_info(b)
    w.pool.batch_end(b)
    o_perm, o_sa, o_ss = op.translate(t2a)
    assert perm.tolist() == o_perm.tolist() and sa.tolist() == o_sa.tolist() and ss.tolist() == o_ss.tolist()
    print("%s: tables and translation match (%d groups)" % (name, len(sa)), flush=True)

    # properties on every slot
    rank_of = np.asarray(w.ranks)[t2a]
    col = np.arange(w.max_rank)[None, :]
    for s in range(lay.n_slots):
        v = w.v[s].cpu().numpy()[:T]
        assert not np.isnan(v).any(), "slot %d: v has unwritten entries" % s
        assert (v[col >= rank_of[:, None]] == 0).all(), "slot %d: v not zero beyond the rank" % s

    # sampled rows: hottest group, a mid group, singletons, first and last token
    ids, counts = np.unique(t2a, return_counts=True)
    order = np.argsort(-counts)
    picks = [ids[order[0]], ids[order[len(order) // 2]], ids[order[-1]], ids[order[-2]]]
    toks = sorted(set([0, T - 1] + [int(np.nonzero(t2a == a)[0][k]) for a in picks for k in (0, -1)]
                      + rng.choice(T, size=n_tok_checked, replace=False).tolist()))
    sel = np.asarray(toks, np.int32)
    slots = sorted(set([0, lay.n_slots - 1] + rng.choice(lay.n_slots, size=min(n_slots_checked, lay.n_slots),
                                                        replace=False).tolist()))
    worst_v = worst_y = 0.0
    for s in slots:
        x, y0 = w.host_x(s), np.ascontiguousarray(w.host_y0(s))
        v_ref = op.shrink(s, x, t2a, acc64=True, tok_sel=sel)
        y_ref = op.expand(s, v_ref, t2a, y0.copy(), acc64=True, tok_sel=sel)
        v_got = w.v[s].cpu().numpy()[:T]
        y_got = torch_to_raw(w.y[s], lay.dtype)[:T]
        ev = rel_err(v_got[sel], v_ref[sel])
        ey = rel_err(from_elt(y_got[sel], lay.dtype), from_elt(y_ref[sel], lay.dtype))
        worst_v, worst_y = max(worst_v, ev), max(worst_y, ey)
        assert ev <= TOL_V, "slot %d: v error %.3g" % (s, ev)
        assert ey <= TOL_Y[lay.dtype], "slot %d: y error %.3g" % (s, ey)
    print("%s: %d slots x %d tokens sampled, worst err_v %.3g err_y %.3g" % (name, len(slots), len(sel), worst_v, worst_y),
          flush=True)
    op.close()
    w.close()


def test_cfg1_decode_7b_full_size(oracle_mod):
    _run(oracle_mod, "cfg1", 6, 10)


def test_cfg2_prefill_full_size(oracle_mod):
    _run(oracle_mod, "cfg2", 4, 24)


def test_cfg4_decode_13b_layer_full_size(oracle_mod):
    _run(oracle_mod, "cfg4", 6, 10)


def test_cfg5_decode_gqa_projections_full_size(oracle_mod):
    _run(oracle_mod, "cfg5", 6, 10)
