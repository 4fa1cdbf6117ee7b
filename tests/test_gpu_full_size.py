"""Full-size workloads in the launch configuration bench.py times, checked element by element.

The oracle runs the whole step on all host threads (fp64 accumulation, OpenMP over tokens) through
its own page pool holding the same adapters: every element of v and of y of every slot is compared,
page tables and the batch translation are compared in full, and v must be zero beyond each token's
rank and y untouched for tokens without adapter.
"""
import time

import numpy as np
import pytest

from workload import from_elt
from helpers import TOL_V, TOL_Y, rel_err, torch_to_raw

pytestmark = pytest.mark.gpu


def _run(oracle_mod, name, slots_per_call=0, options=()):
    import torch
    import bench
    t0 = time.time()
    w = bench.GpuWorkload(name, verbose=True)
    for key, value in options:
        w.pool.set_option(key, value)
    lay, cfg = w.lay, w.cfg
    rng = np.random.default_rng(cfg["seed"] + 7)
    t2a = bench.draw_batch(cfg, rng, w.n_ad)
    T = len(t2a)
    w.alloc_activations(T, cfg["seed"] + 9)
    print("%s: built in %.1fs, T=%d" % (name, time.time() - t0, T), flush=True)
    # poison v so that unwritten entries show
    for v in w.v:
        v.fill_(float("nan"))
    w.step(t2a, slots_per_call or lay.n_slots)  # one call over all slots, as bench.py does by default
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

    from oracle.pool import max_threads
    threads = max_threads()
    rank_of = np.asarray(w.ranks)[t2a]
    col = np.arange(w.max_rank)[None, :]
    worst_v = worst_y = 0.0
    t0 = time.time()
    for s in range(lay.n_slots):
        v_got = w.v[s].cpu().numpy()[:T]
        assert not np.isnan(v_got).any(), "slot %d: v has unwritten entries" % s
        assert (v_got[col >= rank_of[:, None]] == 0).all(), "slot %d: v not zero beyond the rank" % s
        x, y0 = w.host_x(s), np.ascontiguousarray(w.host_y0(s))
        v_ref = op.shrink(s, x, t2a, acc64=True, threads=threads)
        y_ref = op.expand(s, v_ref, t2a, y0.copy(), acc64=True, threads=threads)
        y_got = torch_to_raw(w.y[s], lay.dtype)[:T]
        ev = rel_err(v_got, v_ref)
        ey = rel_err(from_elt(y_got, lay.dtype), from_elt(y_ref, lay.dtype))
        worst_v, worst_y = max(worst_v, ev), max(worst_y, ey)
        assert ev <= TOL_V, "slot %d: v error %.3g" % (s, ev)
        assert ey <= TOL_Y[lay.dtype], "slot %d: y error %.3g" % (s, ey)
        if s % 16 == 15:
            print("%s: slots 0..%d checked (%.1fs)" % (name, s, time.time() - t0), flush=True)
    print("%s: every element of %d slots x %d tokens checked in %.1fs on %d threads, worst err_v %.3g err_y %.3g" % (
        name, lay.n_slots, T, time.time() - t0, threads, worst_v, worst_y), flush=True)
    op.close()
    w.close()


def test_cfg1_decode_7b_full_size(oracle_mod):
    _run(oracle_mod, "cfg1")


def test_cfg1_decode_7b_one_layer_per_call(oracle_mod):
    """The same step as a decoder would issue it: one call per layer (q, k, v, o = 4 slots)."""
    _run(oracle_mod, "cfg1", slots_per_call=4)


def test_cfg2_prefill_full_size(oracle_mod):
    _run(oracle_mod, "cfg2")


def test_cfg2_prefill_full_size_panel_workgroups_of_512_columns(oracle_mod):
    """The form of the panel kernel that launches of more than 8192 workgroups take (a 4-slot call has fewer)."""
    _run(oracle_mod, "cfg2", options=(("panel_half_max_workgroups", 0),))


def test_cfg4_decode_13b_layer_full_size(oracle_mod):
    _run(oracle_mod, "cfg4")


def test_cfg5_decode_gqa_projections_full_size(oracle_mod):
    _run(oracle_mod, "cfg5")
