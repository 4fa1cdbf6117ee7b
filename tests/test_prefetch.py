"""Prefetch manager (Sec. III-B "Proactive Prefetching") on placement-only pools and on the oracle's pool.

Threshold rule p_hat > theta, never evicting a predicted adapter, and the synthetic predictor that
stands in for the paper's LSTM.  The policy's numbers are this build's reading: parity is unpinned
beyond "the same decisions give the same page tables on both sides".
"""
import numpy as np

from workload import CONFIGS, churn_trace, config_layout, draw_ranks, zipf_probs


class _Wrap:
    def __init__(self, pool):
        self.pool, self.tables = pool, {}

    def load(self, aid, rank, scale, blob, stream=None):
        self.tables[aid] = self.pool.load(aid, rank, scale, blob)

    def evict(self, aid):
        self.pool.evict(aid)
        del self.tables[aid]


def _setup(pop, n_pages, seed=3):
    import paper_2512_20210_amd as B
    cfg = CONFIGS["cfg3"]
    lay = config_layout(cfg)
    ranks = draw_ranks(np.random.default_rng(seed), pop, cfg["rank_choices"])
    scales = [16.0 / r for r in ranks]
    g = _Wrap(B.PagedLoraPool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128, placement_only=True))
    return cfg, lay, ranks, scales, g


def test_predictor_quality_is_recall_and_precision():
    from paper_2512_20210_amd.prefetch import SyntheticPredictor
    pop = 1024
    popularity = zipf_probs(pop, 1.0)
    rng = np.random.default_rng(0)
    for q in (0.0, 0.5, 0.86, 1.0):
        pred = SyntheticPredictor(pop, popularity, q, theta=0.5, seed=1)
        tp = fn = fp = 0
        for _ in range(200):
            win = rng.choice(pop, size=100, p=popularity)
            need = set(np.unique(win).tolist())
            p_hat = pred.predict(win)
            assert p_hat.shape == (pop,) and (p_hat > 0).all() and (p_hat <= 1).all()
            flagged = set(np.nonzero(p_hat > 0.5)[0].tolist())
            assert len(flagged) == len(need)      # one wrong adapter for every missed one
            tp += len(flagged & need)
            fn += len(need - flagged)
            fp += len(flagged - need)
        recall, precision = tp / (tp + fn), tp / (tp + fp)
        assert abs(recall - q) < 0.02 and abs(precision - q) < 0.02, (q, recall, precision)


def test_perfect_prediction_removes_cold_starts_when_the_interval_fits():
    from paper_2512_20210_amd.prefetch import PrefetchManager, SyntheticPredictor
    pop, n_pages = 512, 8192                       # 512 MiB of 64 KiB pages: several intervals fit
    cfg, lay, ranks, scales, g = _setup(pop, n_pages)
    popularity = zipf_probs(pop, 1.0)
    pred = SyntheticPredictor(pop, popularity, 1.0, seed=5)
    m = PrefetchManager(g, ranks, scales, lambda i: None, theta=0.5)
    trace = churn_trace(np.random.default_rng(4), 3000, pop, 1.0, burst_prob=0.0)   # 100 requests per interval
    for win in trace:
        started = m.begin_interval(pred.predict(win))
        assert all(i in m.resident() for i in started)
        for aid in win:
            assert m.request(int(aid)), "a perfectly predicted adapter must be in memory when it is requested"
    assert m.cold_starts == 0 and m.failed == 0 and m.prefetch_no_room == 0
    assert m.useful_prefetches == m.prefetch_loads - len(m.prefetched) - m.wasted_prefetches
    assert m.wasted_prefetches == 0               # every prefetched adapter was requested in its interval
    g.pool.close()


def test_prefetch_never_evicts_a_predicted_adapter_and_stops_when_out_of_room():
    from paper_2512_20210_amd.prefetch import PrefetchManager
    pop, n_pages = 64, 64 * 6                      # rank 8 = 8 pages of 64 KiB (4 slots 4096->4096): room for 48 adapters
    cfg, lay, _, _, g = _setup(pop, n_pages)
    ranks, scales = [8] * pop, [1.0] * pop
    m = PrefetchManager(g, ranks, scales, lambda i: None, theta=0.5)
    for aid in range(48):
        m.request(aid)
    assert g.pool.stats()["free_pages"] == 0
    p_hat = np.full(pop, 0.1)
    p_hat[0:40] = 0.9                              # 40 residents are predicted, 8 are not
    p_hat[48:64] = 0.8                             # 16 absent adapters are predicted
    started = m.begin_interval(p_hat)
    assert started == list(range(48, 56))          # only the 8 unpredicted residents could give way
    assert m.prefetch_no_room == 1 and all(i in m.resident() for i in range(40))
    assert not any(i in m.resident() for i in range(40, 48))
    # a prefetched adapter that is evicted before any request counts as wasted
    for aid in range(56, 64):
        m.request(aid)                             # on demand: evicts by score, predicted or not
    assert m.wasted_prefetches + len(m.prefetched) + m.useful_prefetches == m.prefetch_loads
    g.pool.close()


def test_same_prefetch_decisions_same_tables_on_oracle_and_library(oracle_mod):
    from paper_2512_20210_amd.prefetch import PrefetchManager, SyntheticPredictor
    pop, n_pages = 512, 2048
    cfg, lay, ranks, scales, g = _setup(pop, n_pages)
    o = _Wrap(oracle_mod.OraclePool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128))
    zero = {int(r): np.zeros(lay.adapter_elems(int(r)), np.uint16) for r in set(ranks.tolist())}
    popularity = zipf_probs(pop, 1.0)
    pred = SyntheticPredictor(pop, popularity, 0.86, seed=6)
    mg = PrefetchManager(g, ranks, scales, lambda i: None)
    mo = PrefetchManager(o, ranks, scales, lambda i: zero[int(ranks[i])])
    for win in churn_trace(np.random.default_rng(4), 3000, pop, 1.0):
        p_hat = pred.predict(win)
        assert mg.begin_interval(p_hat) == mo.begin_interval(p_hat)
        for aid in win:
            assert mg.request(int(aid)) == mo.request(int(aid))
    assert mg.log == mo.log and mg.evictions > 100 and mg.prefetch_loads > 100
    assert sorted(g.tables) == sorted(o.tables)
    for aid in g.tables:
        assert g.tables[aid].tolist() == o.tables[aid].tolist()
    g.pool.close()


def test_cold_start_rate_falls_with_prediction_quality():
    from paper_2512_20210_amd.prefetch import PrefetchManager, SyntheticPredictor
    pop, n_pages = 2048, 16384                     # 1 GiB pool, 1-layer adapters of the churn workload
    rates = {}
    for q in (None, 0.5, 0.86, 1.0):
        cfg, lay, ranks, scales, g = _setup(pop, n_pages)
        popularity = zipf_probs(pop, 1.0)
        m = PrefetchManager(g, ranks, scales, lambda i: None)
        pred = SyntheticPredictor(pop, popularity, q, seed=7) if q is not None else None
        n = 0
        for win in churn_trace(np.random.default_rng(8), 6000, pop, 1.0, burst_prob=0.1, burst_mult=8):
            if pred is not None:
                m.begin_interval(pred.predict(win))
            for aid in win:
                m.request(int(aid))
                n += 1
        rates[q] = m.cold_starts / n
        g.pool.close()
    assert rates[1.0] < 0.02 < rates[None]
    assert rates[1.0] < rates[0.86] < rates[0.5] < rates[None]
    assert rates[0.86] < 0.5 * rates[None]          # the paper's 68 % cold-start reduction (Sec. V-B) is of this order
