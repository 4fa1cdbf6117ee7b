"""The library's residency policy (plora_manager_*: Sec. III-B, Eq. 3 and "Proactive Prefetching") against
the policy oracle: the same requests and predictions must give the same hits, the same loads and
evictions in the same order, bit-identical scores, the same counters, and therefore the same page
tables.  The library runs on a placement-only pool (no GPU), the oracle on its own pool.
"""
import numpy as np
import pytest

from workload import CONFIGS, SyntheticPredictor, churn_trace, config_layout, draw_ranks, zipf_probs


def _both(oracle_mod, pop, n_pages, seed=3, ranks=None, **kw):
    import paper_2512_20210_amd as B
    cfg = CONFIGS["cfg3"]
    lay = config_layout(cfg)
    ranks = draw_ranks(np.random.default_rng(seed), pop, cfg["rank_choices"]) if ranks is None else ranks
    scales = [16.0 / r for r in ranks]
    g = B.PagedLoraPool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128, placement_only=True)
    o = oracle_mod.OraclePool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128)
    mg = B.ResidencyManager(g, ranks, scales, **kw)
    mo = oracle_mod.OracleManager(o, pop, **kw)
    zero = {int(r): np.zeros(lay.adapter_elems(int(r)), np.uint16) for r in set(int(x) for x in ranks)}
    for i, r in enumerate(ranks):
        mo.set_adapter(i, int(r), scales[i], zero[int(r)])
    return g, o, mg, mo, ranks


def _same_state(g, o, mg, mo):
    st = mg.stats()
    for k in ("hits", "misses", "loads", "evictions", "failed_loads", "prefetch_loads", "useful_prefetches",
              "wasted_prefetches", "prefetch_no_room"):
        assert st[k] == getattr(mo, k), k
    assert st["skipped_busy"] == 0
    assert mg.log() == mo.log
    assert mg.residents().tolist() == mo.residents()
    sg, so = mg.scores(), mo.scores()
    assert sg == so                                         # doubles, bit for bit
    assert st["util_samples"] == len(mo.byte_util)
    if mo.byte_util:
        assert st["byte_util_min"] == min(mo.byte_util) and st["page_util_min"] == min(mo.page_util)
        assert abs(st["byte_util_sum"] - sum(mo.byte_util)) < 1e-9 * len(mo.byte_util)
    ps, os_ = g.stats(), o.stats()
    for k in ("used_pages", "free_pages", "resident_bytes", "loads", "evictions"):
        assert ps[k] == os_[k], k


@pytest.mark.parametrize("weights", [(0.4, 0.3, 0.3), (1.0, 0.0, 0.0), (0.0, 1.0, 0.0), (0.0, 0.0, 0.0), (0.2, 0.7, 0.1)])
def test_on_demand_decisions_match_the_oracle(oracle_mod, weights):
    pop, n_pages = 512, 2048
    a, b, c = weights
    g, o, mg, mo, ranks = _both(oracle_mod, pop, n_pages, alpha=a, beta=b, gamma=c, window=300)
    popularity = zipf_probs(pop, 1.0)
    mg.set_prediction(popularity / popularity.max())
    mo.p_hat = (popularity / popularity.max()).astype(np.float32)
    n = 0
    for win in churn_trace(np.random.default_rng(4), 3000, pop, 1.0):
        for aid in win:
            assert mg.request(int(aid)) == mo.request(int(aid)), "request %d (adapter %d)" % (n, aid)
            n += 1
        _same_state(g, o, mg, mo)
    assert mo.evictions > 100
    assert min(mo.byte_util) >= 0.87                        # the >= 87 % target of Sec. V-D on byte utilisation
    # the tables themselves: reload one evicted adapter on both sides
    victim = mo.residents()[0]
    g.evict(victim)
    o.evict(victim)
    assert g.load(victim, int(ranks[victim]), 1.0, None).tolist() == o.load(victim, int(ranks[victim]), 1.0,
                                                                            np.zeros(config_layout(CONFIGS["cfg3"]).adapter_elems(int(ranks[victim])), np.uint16)).tolist()
    mg.close()
    g.close()


@pytest.mark.parametrize("quality", [0.5, 0.86, 1.0])
def test_prefetch_decisions_match_the_oracle(oracle_mod, quality):
    pop, n_pages = 512, 2048
    g, o, mg, mo, ranks = _both(oracle_mod, pop, n_pages)
    pred = SyntheticPredictor(pop, zipf_probs(pop, 1.0), quality, seed=6)
    for win in churn_trace(np.random.default_rng(4), 3000, pop, 1.0):
        p_hat = pred.predict(win).astype(np.float32)
        started = mo.prefetch(p_hat)
        assert mg.prefetch(p_hat) == len(started)
        for aid in win:
            assert mg.request(int(aid)) == mo.request(int(aid))
        _same_state(g, o, mg, mo)
        for aid in started[:5]:
            assert mg.state(aid) & 1 == (aid in mo.last_use) and bool(mg.state(aid) & 2) == (aid in mo.prefetched)
    assert mo.evictions > 100 and mo.prefetch_loads > 100
    mg.close()
    g.close()


def test_hand_worked_example_through_the_library(oracle_mod):
    """The four-adapter example of tests/test_oracle_manager.py (scores 0.5667, 0.15, 0.2833, 0.55; adapter 2
    goes once adapter 1 is predicted), asked of the library directly."""
    import paper_2512_20210_amd as B
    g = B.PagedLoraPool(4096, 4, [64], [64], B.PLORA_BF16, 8, 64, placement_only=True)
    m = B.ResidencyManager(g, [16] * 8, [1.0] * 8)
    for aid in (0, 1, 2, 0, 3):
        m.request(aid)
    assert m.scores() == {0: (0.4 * (2 / 3) + 0.3 * 1.0) + 0.0, 1: (0.4 * 0.0 + 0.3 * 0.5) + 0.0,
                          2: (0.4 * (1 / 3) + 0.3 * 0.5) + 0.0, 3: (0.4 * 1.0 + 0.3 * 0.5) + 0.0}
    m.set_prediction(np.array([0, 1, 0, 0, 0, 0, 0, 0], np.float32))
    assert m.request(4) is False
    assert m.log()[-2:] == [(1, 2), (0, 4)] and m.residents().tolist() == [0, 1, 3, 4]
    m.close()
    g.close()


def test_manager_argument_checks():
    import paper_2512_20210_amd as B
    g = B.PagedLoraPool(4096, 4, [64], [64], B.PLORA_BF16, 8, 64, placement_only=True)
    assert B.plora_manager_create(g.h, 0)[0] == B.PLORA_ERR_INVAL
    assert B.plora_manager_create(g.h, 8, alpha=-1.0)[0] == B.PLORA_ERR_INVAL
    assert B.plora_manager_create(g.h, 8, theta=1.5)[0] == B.PLORA_ERR_INVAL
    assert B.plora_manager_create(g.h, 8, window=0)[0] == B.PLORA_ERR_INVAL
    rc, h = B.plora_manager_create(g.h, 8)
    assert rc == B.PLORA_OK
    assert B.plora_manager_request(h, 3)[0] == B.PLORA_ERR_INVAL          # not registered
    assert B.plora_manager_set_adapter(h, 9, 16, 1.0) == B.PLORA_ERR_INVAL
    assert B.plora_manager_set_adapter(h, 3, 16, 1.0) == B.PLORA_OK
    assert B.plora_manager_request(h, 3) == (B.PLORA_OK, 0)
    assert B.plora_manager_request(h, 3) == (B.PLORA_OK, 1)
    assert B.plora_manager_set_adapter(h, 3, 8, 1.0) == B.PLORA_ERR_BUSY  # resident
    assert B.plora_manager_destroy(h) == B.PLORA_OK
    g.close()
