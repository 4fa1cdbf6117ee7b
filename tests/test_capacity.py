"""Pool utilisation under churn (Sec. V-D: > 87 % for page-based allocation) on placement-only pools.

The paged allocator never fails while enough pages are free (no external fragmentation, Sec. III-C);
a contiguous first-fit block allocator over the same byte budget does, and ends up less full.
The eviction policy is this build's reading of Eq. 3 (parity unpinned).
"""
import numpy as np

from workload import CONFIGS, churn_trace, draw_ranks


def _run(alloc, page_bytes, n_slots, pop, n_events=4000):
    from paper_2512_20210_amd.capacity import utilisation_under_trace
    cfg = CONFIGS["cfg3"]
    ranks = draw_ranks(np.random.default_rng(cfg["seed"]), pop, cfg["rank_choices"])
    trace = churn_trace(np.random.default_rng(cfg["seed"] + 1), n_events, pop, cfg["zipf"], cfg["window"],
                        cfg["burst_prob"], cfg["burst_mult"])
    d = [4096] * n_slots
    return utilisation_under_trace(d, d, cfg["dtype"], page_bytes, cfg["n_pages"] * cfg["page_bytes"], ranks, trace,
                                   n_events, alloc)


def test_paged_pool_stays_above_87_percent_and_never_fragments():
    for n_slots, pop in ((4, 4096), (128, 256)):
        r = _run("pages", 64 << 10, n_slots, pop)
        assert r["evictions"] > 100 and r["failed"] == 0
        assert r["nomem_with_free_space"] == 0
        assert r["byte_util_min"] >= 0.87, r


def test_block_allocator_fragments_and_fills_less():
    p = _run("pages", 64 << 10, 128, 256)
    b = _run("block", 256, 128, 256)
    assert b["nomem_with_free_space"] > 0                 # external fragmentation
    assert b["byte_util_avg"] < p["byte_util_avg"] and b["byte_util_min"] < p["byte_util_min"]


def test_large_pages_trade_internal_fragmentation():
    """2 MiB pages (the paper's default) with 256 KiB ... 8 MiB adapters: pages fill up, bytes do not."""
    r = _run("pages", 2 << 20, 4, 4096)
    assert r["alloc_util_avg"] > 0.99 and r["byte_util_avg"] < 0.87
