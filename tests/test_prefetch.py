"""Threshold prefetching (Sec. III-B "Proactive Prefetching") through the library's policy on placement-only
pools: what the rule achieves on synthetic predictions of chosen quality, and the synthetic predictor
itself (an input generator).  Decision parity with the oracle is in tests/test_manager.py.
"""
import numpy as np

from workload import CONFIGS, SyntheticPredictor, churn_trace, config_layout, draw_ranks, zipf_probs


def _setup(pop, n_pages, seed=3, ranks=None):
    import paper_2512_20210_amd as B
    cfg = CONFIGS["cfg3"]
    lay = config_layout(cfg)
    ranks = draw_ranks(np.random.default_rng(seed), pop, cfg["rank_choices"]) if ranks is None else ranks
    g = B.PagedLoraPool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128, placement_only=True)
    return g, B.ResidencyManager(g, ranks, [16.0 / r for r in ranks])


def test_predictor_quality_is_recall_and_precision():
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
    pop, n_pages = 512, 8192                       # 512 MiB of 64 KiB pages: several intervals fit
    g, m = _setup(pop, n_pages)
    pred = SyntheticPredictor(pop, zipf_probs(pop, 1.0), 1.0, seed=5)
    for win in churn_trace(np.random.default_rng(4), 3000, pop, 1.0, burst_prob=0.0):   # 100 requests per interval
        m.prefetch(pred.predict(win))
        for aid in win:
            assert m.request(int(aid)), "a perfectly predicted adapter must be in memory when it is requested"
    st = m.stats()
    assert st["misses"] == 0 and st["failed_loads"] == 0 and st["prefetch_no_room"] == 0
    assert st["wasted_prefetches"] == 0            # every prefetched adapter was requested in its interval
    assert st["useful_prefetches"] == st["prefetch_loads"]
    m.close()
    g.close()


def test_prefetch_never_evicts_a_predicted_adapter_and_stops_when_out_of_room():
    pop, n_pages = 64, 64 * 6                      # rank 8 = 8 pages of 64 KiB (4 slots 4096->4096): room for 48 adapters
    g, m = _setup(pop, n_pages, ranks=[8] * pop)
    for aid in range(48):
        m.request(aid)
    assert g.stats()["free_pages"] == 0
    p_hat = np.full(pop, 0.1, np.float32)
    p_hat[0:40] = 0.9                              # 40 residents are predicted, 8 are not
    p_hat[48:64] = 0.8                             # 16 absent adapters are predicted
    assert m.prefetch(p_hat) == 8                  # only the 8 unpredicted residents could give way
    res = set(m.residents().tolist())
    assert m.stats()["prefetch_no_room"] == 1 and res == set(range(40)) | set(range(48, 56))
    for aid in range(56, 64):
        m.request(aid)                             # on demand: evicts by score, predicted or not
    st = m.stats()
    n_still = sum(1 for i in range(pop) if m.state(i) & 2)
    assert st["wasted_prefetches"] + n_still + st["useful_prefetches"] == st["prefetch_loads"]
    m.close()
    g.close()


def test_cold_start_rate_falls_with_prediction_quality():
    pop, n_pages = 2048, 16384                     # 1 GiB pool, 1-layer adapters of the churn workload
    rates = {}
    for q in (None, 0.5, 0.86, 1.0):
        g, m = _setup(pop, n_pages)
        pred = SyntheticPredictor(pop, zipf_probs(pop, 1.0), q, seed=7) if q is not None else None
        n = 0
        for win in churn_trace(np.random.default_rng(8), 6000, pop, 1.0, burst_prob=0.1, burst_mult=8):
            if pred is not None:
                m.prefetch(pred.predict(win))
            for aid in win:
                m.request(int(aid))
                n += 1
        rates[q] = m.stats()["misses"] / n
        m.close()
        g.close()
    assert rates[1.0] < 0.02 < rates[None]
    assert rates[1.0] < rates[0.86] < rates[0.5] < rates[None]
    assert rates[0.86] < 0.5 * rates[None]          # the paper's 68 % cold-start reduction (Sec. V-B) is of this order
