"""Residency manager (eviction score of Sec. III-B, Eq. 3) on a placement-only pool and on the oracle.

The score's weights and normalisation are this build's reading (the paper gives none): parity is
unpinned beyond "both pools see the same decisions and end with the same page tables".
"""
import numpy as np

from workload import CONFIGS, DT_BF16, Layout, churn_trace, config_layout, draw_ranks


class _Wrap:
    def __init__(self, pool):
        self.pool, self.tables = pool, {}

    def load(self, aid, rank, scale, blob, stream=None):
        self.tables[aid] = self.pool.load(aid, rank, scale, blob)

    def evict(self, aid):
        self.pool.evict(aid)
        del self.tables[aid]


def test_same_decisions_same_tables_and_utilisation(oracle_mod):
    import paper_2512_20210_amd as B
    from paper_2512_20210_amd.manager import ResidencyManager
    cfg = CONFIGS["cfg3"]
    lay = config_layout(cfg)
    pop, n_pages = 512, 2048
    rng = np.random.default_rng(3)
    ranks = draw_ranks(rng, pop, cfg["rank_choices"])
    scales = [16.0 / r for r in ranks]
    g = _Wrap(B.PagedLoraPool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128, placement_only=True))
    o = _Wrap(oracle_mod.OraclePool(cfg["page_bytes"], n_pages, lay.d_in, lay.d_out, lay.dtype, pop, 128))
    zero = {int(r): np.zeros(lay.adapter_elems(int(r)), np.uint16) for r in set(ranks.tolist())}
    mg = ResidencyManager(g, ranks, scales, lambda i: None)
    mo = ResidencyManager(o, ranks, scales, lambda i: zero[int(ranks[i])])
    util = []
    n = 0
    for win in churn_trace(np.random.default_rng(4), 4000, pop, 1.0):
        for aid in win:
            hg, ho = mg.request(int(aid)), mo.request(int(aid))
            assert hg == ho
            n += 1
            if mg.evictions:
                st = g.pool.stats()
                util.append(st["resident_bytes"] / (st["n_pages"] * st["page_bytes"]))
    assert mg.log == mo.log and mg.evictions > 100
    assert sorted(g.tables) == sorted(o.tables)
    for aid in g.tables:
        assert g.tables[aid].tolist() == o.tables[aid].tolist()
    assert min(util) >= 0.87
    g.pool.close()


def test_score_orders_by_recency_frequency_and_prediction():
    from paper_2512_20210_amd.manager import ResidencyManager

    class Never:
        def load(self, *a):
            pass

        def evict(self, aid):
            pass
    ranks, scales = [8] * 4, [1.0] * 4
    m = ResidencyManager(Never(), ranks, scales, lambda i: None, alpha=1.0, beta=0.0, gamma=0.0)
    for aid in (0, 1, 2, 3, 0):
        m.request(aid)
    sc = m.scores()
    assert sc[0] == 1.0 and sc[1] == 0.0 and sc[1] < sc[2] < sc[3] < sc[0]   # 1 is the least recently used
    m = ResidencyManager(Never(), ranks, scales, lambda i: None, alpha=0.0, beta=1.0, gamma=0.0)
    for aid in (0, 1, 1, 1, 2, 2, 3):
        m.request(aid)
    sc = m.scores()
    assert sc[1] == 1.0 and abs(sc[2] - 2 / 3) < 1e-12 and sc[0] == sc[3] == 1 / 3
    m = ResidencyManager(Never(), ranks, scales, lambda i: None, alpha=0.0, beta=0.0, gamma=1.0, p_hat=[0.1, 0.9, 0.5, 0.2])
    for aid in range(4):
        m.request(aid)
    assert min(m.scores(), key=m.scores().get) == 0
