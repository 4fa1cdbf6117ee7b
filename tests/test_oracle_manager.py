"""Pins of the policy oracle (oracle/manager.py): hand-worked examples of the eviction score (Sec. III-B,
Eq. 3) and of the prefetch rule under the reading stated in that file.  Every expected value below was
worked out by hand from the reading (the arithmetic is in the comments); none comes from the library.
The paper itself prints no worked example of Eq. 3 (it gives neither weights nor normalisation), so
what is pinned is the reading, term by term: a swapped term, a wrong direction, a wrong tie rule or
a window that does not slide fails one of these.
"""
import numpy as np
import pytest

from workload import DT_BF16


def _pool(oracle_mod, n_pages, n_adapters=8):
    # one slot 64 -> 64, bf16: a rank-16 adapter is 16 * 2 * 128 = 4096 bytes = exactly one 4 KiB page
    return oracle_mod.OraclePool(4096, n_pages, [64], [64], DT_BF16, n_adapters, 64)


def _mgr(oracle_mod, n_pages, ranks=None, **kw):
    ranks = ranks or [16] * 8
    pool = _pool(oracle_mod, n_pages, len(ranks))
    m = oracle_mod.OracleManager(pool, len(ranks), **kw)
    for i, r in enumerate(ranks):
        m.set_adapter(i, r, 1.0, np.zeros(r * 128, np.uint16))
    return m


def test_recency_term_alone(oracle_mod):
    m = _mgr(oracle_mod, 8, alpha=1.0, beta=0.0, gamma=0.0)
    for aid in (0, 1, 2, 3, 0):
        m.request(aid)
    # last requests at clocks 0 -> 5, 1 -> 2, 2 -> 3, 3 -> 4: oldest first 1, 2, 3, 0 -> k / 3
    assert m.scores() == {0: 1.0, 1: 0.0, 2: 1 / 3, 3: 2 / 3}
    one = _mgr(oracle_mod, 8, alpha=1.0, beta=0.0, gamma=0.0)
    one.request(5)
    assert one.scores() == {5: 1.0}                       # a lone resident


def test_frequency_term_alone_and_its_sliding_window(oracle_mod):
    m = _mgr(oracle_mod, 8, alpha=0.0, beta=1.0, gamma=0.0)
    for aid in (0, 1, 1, 1, 2, 2, 3):
        m.request(aid)
    # counts 1, 3, 2, 1 over the largest, 3
    assert m.scores() == {0: 1 / 3, 1: 1.0, 2: 2 / 3, 3: 1 / 3}
    m = _mgr(oracle_mod, 8, alpha=0.0, beta=1.0, gamma=0.0, window=4)
    for aid in (0, 1, 1, 1, 2, 2, 3):
        m.request(aid)
    # only the last four requests count: 1, 2, 2, 3 -> counts 0, 1, 2, 1 over 2
    assert m.scores() == {0: 0.0, 1: 0.5, 2: 1.0, 3: 0.5}


def test_prediction_term_alone(oracle_mod):
    m = _mgr(oracle_mod, 8, alpha=0.0, beta=0.0, gamma=1.0)
    for aid in range(4):
        m.request(aid)
    assert m.scores() == {0: 0.0, 1: 0.0, 2: 0.0, 3: 0.0}  # no prediction yet: p_hat = 0
    m.p_hat = np.array([0.125, 0.875, 0.5, 0.25, 0, 0, 0, 0], np.float32)
    assert m.scores() == {0: 0.125, 1: 0.875, 2: 0.5, 3: 0.25}


def test_combined_score_and_eviction_order(oracle_mod):
    m = _mgr(oracle_mod, 4)                                # default weights 0.4, 0.3, 0.3; room for four adapters
    for aid in (0, 1, 2, 0, 3):
        m.request(aid)
    # last use 0 -> 4, 1 -> 2, 2 -> 3, 3 -> 5: oldest first 1, 2, 0, 3 -> LRU 0, 1/3, 2/3, 1
    # counts 2, 1, 1, 1 over 2 -> freq 1, .5, .5, .5
    want = {0: (0.4 * (2 / 3) + 0.3 * 1.0) + 0.0, 1: (0.4 * 0.0 + 0.3 * 0.5) + 0.0,
            2: (0.4 * (1 / 3) + 0.3 * 0.5) + 0.0, 3: (0.4 * 1.0 + 0.3 * 0.5) + 0.0}
    assert m.scores() == want
    assert [round(want[i], 4) for i in range(4)] == [0.5667, 0.15, 0.2833, 0.55]
    # a prediction for adapter 1 lifts it over adapter 2: .15 + .3 = .45 > .2833
    m.p_hat = np.array([0, 1, 0, 0, 0, 0, 0, 0], np.float32)
    assert min(m.scores(), key=m.scores().get) == 2
    # the pool is full: a request for adapter 4 evicts the lowest score, adapter 2, and nothing else
    assert m.request(4) is False
    assert m.log[-2:] == [(1, 2), (0, 4)] and m.residents() == [0, 1, 3, 4]
    # without the prediction it would have been adapter 1
    m2 = _mgr(oracle_mod, 4)
    for aid in (0, 1, 2, 0, 3, 4):
        m2.request(aid)
    assert m2.log[-2:] == [(1, 1), (0, 4)]
    # a larger adapter takes as many victims as it needs, in score order: rank 32 = two pages
    m3 = _mgr(oracle_mod, 4, ranks=[16, 16, 16, 16, 32, 16, 16, 16])
    for aid in (0, 1, 2, 0, 3, 4):
        m3.request(aid)
    assert m3.log[-3:] == [(1, 1), (1, 2), (0, 4)]        # .15, then .2833
    assert m3.evictions == 2 and m3.loads == 5 and m3.misses == 5 and m3.hits == 1


def test_equal_scores_go_by_lowest_id_and_equal_clocks_by_id(oracle_mod):
    m = _mgr(oracle_mod, 4, alpha=0.0, beta=0.0, gamma=0.0)
    for aid in (3, 2, 1, 0):
        m.request(aid)
    m.request(7)
    assert m.log[-2:] == [(1, 0), (0, 7)]                  # all scores 0: the lowest id goes
    # adapters prefetched in one round share a clock value: their recency order is by id
    m = _mgr(oracle_mod, 8, alpha=1.0, beta=0.0, gamma=0.0)
    m.request(6)
    p = np.zeros(8, np.float32)
    p[[5, 2]] = 0.75, 0.75
    assert m.prefetch(p) == [2, 5]                         # equal probabilities: by id
    # clocks 6 -> 1, 2 -> 1, 5 -> 1: oldest first 2, 5, 6
    assert m.scores() == {2: 0.0, 5: 0.5, 6: 1.0}


def test_prefetch_rule(oracle_mod):
    m = _mgr(oracle_mod, 4, ranks=[16] * 10, theta=0.5)
    for aid in range(4):
        m.request(aid)                                     # pool full: 0, 1, 2, 3
    p = np.full(10, 0.125, np.float32)
    p[[0, 1]] = 0.875                                      # two residents are predicted ...
    p[[4, 5, 6]] = 0.75, 0.9375, 0.625                     # ... and three absent adapters, 5 most probable
    p[7] = 0.5                                             # exactly theta: not predicted
    started = m.prefetch(p)
    # only the unpredicted residents 2 and 3 may give way: 5, then 4 are loaded, 6 finds no room
    assert started == [5, 4] and m.prefetch_no_room == 1
    assert m.residents() == [0, 1, 4, 5] and m.prefetched == {4, 5}
    # victims in score order: 2 (used before 3, equal frequency, equal p_hat) first
    assert m.log[4:] == [(1, 2), (0, 5), (1, 3), (0, 4)]
    assert m.request(5) is True and m.useful_prefetches == 1 and m.prefetched == {4}
    # on demand, a predicted adapter may be evicted; an unrequested prefetched one then counts as wasted
    for aid in (8, 9, 2, 3):
        m.request(aid)
    assert m.wasted_prefetches == 1                        # adapter 4 left without having been requested
    assert m.prefetch_loads == m.useful_prefetches + m.wasted_prefetches + len(m.prefetched)
    assert m.hits + m.misses == 4 + 1 + 4 and m.loads == m.misses + m.prefetch_loads - m.failed_loads
    st = m.pool.stats()
    assert st["loads"] == m.loads and st["evictions"] == m.evictions
    assert len(m.residents()) == st["used_pages"]


def test_utilisation_is_sampled_after_loads_once_the_pool_has_filled(oracle_mod):
    m = _mgr(oracle_mod, 4, ranks=[16, 16, 16, 16, 8, 16, 16, 16])
    for aid in range(4):
        m.request(aid)
    assert m.page_util == []                               # the pool has never refused yet
    m.request(4)                                           # rank 8 = half a page: evicts one, fills half a page
    assert m.page_util == [1.0] and m.byte_util == [3.5 / 4]
