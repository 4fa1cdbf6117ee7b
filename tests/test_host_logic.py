"""Host logic of the library without a GPU: symbols, placement-only pools, batch translation.

The library's allocator and batch translation are integer work: they must match the oracle bit
for bit (page tables, token permutation, group boundaries) over random load / evict histories.
A placement-only pool makes no HIP call, so these run on a machine without a GPU.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from workload import DT_BF16, DT_F16, DT_F32, Layout, draw_tok2adapter

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    import paper_2512_20210_amd as P
    header = open(os.path.join(ROOT, "include", "plora.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(plora_[a-z_0-9]+)\s*\(", header)))
    assert len(names) >= 17
    lib = ctypes.CDLL(P.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "libplora.so does not export %s" % n
        assert hasattr(P, n), "python binding lacks %s" % n
    assert P.plora_version() >= 100


def _pools(oracle_mod, lay, P, n_pages, max_ad, max_rank):
    import paper_2512_20210_amd as B
    o = oracle_mod.OraclePool(P, n_pages, lay.d_in, lay.d_out, lay.dtype, max_ad, max_rank)
    g = B.PagedLoraPool(P, n_pages, lay.d_in, lay.d_out, lay.dtype, max_ad, max_rank, placement_only=True)
    return o, g


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_page_tables_match_oracle_over_random_history(oracle_mod, seed):
    import paper_2512_20210_amd as B
    rng = np.random.default_rng(seed)
    lay = Layout((64, 32), (32, 96), DT_BF16)
    P, n_pages, max_ad, max_rank = 4096, 200, 64, 128
    o, g = _pools(oracle_mod, lay, P, n_pages, max_ad, max_rank)
    resident = {}
    for step in range(1500):
        aid = int(rng.integers(0, max_ad))
        if rng.random() < 0.55:
            rank = int(rng.integers(1, max_rank + 1))
            blob = np.zeros(lay.adapter_elems(rank), np.uint16)
            try:
                pt_o = o.load(aid, rank, 1.0, blob)
                code_o = 0
            except oracle_mod.OracleError as e:
                pt_o, code_o = None, e.code
            rc, pt_g = B.plora_load_adapter(g.h, aid, rank, 1.0, None, None)
            assert rc == code_o, (step, rc, code_o)
            if rc == 0:
                assert pt_g.tolist() == pt_o.tolist()
                resident[aid] = rank
        else:
            try:
                o.evict(aid)
                code_o = 0
            except oracle_mod.OracleError as e:
                code_o = e.code
            assert B.plora_evict(g.h, aid) == code_o
            if code_o == 0:
                resident.pop(aid)
        so, sg = o.stats(), g.stats()
        for k in ("used_pages", "free_pages", "resident_bytes", "loads", "evictions"):
            assert so[k] == sg[k], (step, k)
        assert so["nomem"] == sg["nomem_failures"]
        assert sg["resident_adapters"] == len(resident)
        assert sg["internal_frag_bytes"] == sg["used_pages"] * P - sg["resident_bytes"]
        if step % 100 == 0 and resident:
            ids = np.fromiter(resident.keys(), dtype=np.int32)
            t2a = draw_tok2adapter(rng, int(rng.integers(1, 300)), ids, s=1.0, none_frac=0.1)
            perm_o, sa_o, ss_o = o.translate(t2a)
            b = g.batch_begin(t2a)
            perm, sa, ss = g.batch_info(b)
            g.batch_end(b)
            assert perm.tolist() == perm_o.tolist() and sa.tolist() == sa_o.tolist() and ss.tolist() == ss_o.tolist()
    g.close()


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_compaction_matches_oracle_over_random_history(oracle_mod, seed):
    """plora_compact against the oracle's compaction: the same adapters move to the same pages for the
    same bound, adapters named by an open batch stay where they are (the oracle is told to skip them),
    later loads land on the same pages, and the table handed out at load time is the one rewritten."""
    import paper_2512_20210_amd as B
    rng = np.random.default_rng(seed)
    lay = Layout((64, 32), (32, 96), DT_BF16)
    P, n_pages, max_ad, max_rank = 4096, 200, 64, 128
    o, g = _pools(oracle_mod, lay, P, n_pages, max_ad, max_rank)
    resident = {}
    moved_total = 0
    for step in range(1200):
        aid = int(rng.integers(0, max_ad))
        u = rng.random()
        if u < 0.5:
            rank = int(rng.integers(1, max_rank + 1))
            blob = np.zeros(lay.adapter_elems(rank), np.uint16)
            try:
                pt_o, code_o = o.load(aid, rank, 1.0, blob), 0
            except oracle_mod.OracleError as e:
                pt_o, code_o = None, e.code
            rc, pt_g = B.plora_load_adapter(g.h, aid, rank, 1.0, None, None)
            assert rc == code_o, (step, rc, code_o)
            if rc == 0:
                assert pt_g.tolist() == pt_o.tolist()
                resident[aid] = rank
        elif u < 0.9:
            try:
                o.evict(aid)
                code_o = 0
            except oracle_mod.OracleError as e:
                code_o = e.code
            assert B.plora_evict(g.h, aid) == code_o
            if code_o == 0:
                resident.pop(aid)
        else:
            bound = int(rng.choice([0, 0, 3, 40]))
            batch, pinned = None, []
            if resident and rng.random() < 0.5:  # an open batch holds some adapters in place
                ids = np.fromiter(resident.keys(), dtype=np.int32)
                t2a = rng.choice(ids, size=int(rng.integers(1, 6))).astype(np.int32)
                batch = g.batch_begin(t2a)
                pinned = sorted(set(t2a.tolist()))
            got = g.compact(max_pages=bound)
            want = o.compact(max_pages=bound, skip=pinned)
            assert got == want, (step, got, want)
            moved_total += got[1]
            if batch is not None:
                g.batch_end(batch)
            for k in resident:
                assert g.page_table(k).tolist() == o.page_table(k).tolist(), (step, k)
        so, sg = o.stats(), g.stats()
        for k in ("used_pages", "free_pages", "resident_bytes"):
            assert so[k] == sg[k], (step, k)
    assert moved_total > 50 and g.stats()["compacted_adapters"] == moved_total
    # nothing pinned, no bound: every adapter that ends on consecutive pages is handed to the kernels that way
    g.compact()
    o.compact()
    for k in resident:
        assert g.page_table(k).tolist() == o.page_table(k).tolist()
    assert B.plora_compact(None, None, 0)[0] == B.PLORA_ERR_INVAL
    assert B.plora_adapter_pages(g.h, max_ad, )[0] == B.PLORA_ERR_INVAL
    free_id = next(i for i in range(max_ad) if i not in resident)
    assert B.plora_adapter_pages(g.h, free_id)[0] == B.PLORA_ERR_NOTFOUND
    g.close()


def test_adapter_bytes_and_page_counts_match_layout_formula(oracle_mod):
    import paper_2512_20210_amd as B
    for dtype in (DT_F16, DT_BF16, DT_F32):
        lay = Layout((1024, 5120), (1024, 13824), dtype)
        o, g = _pools(oracle_mod, lay, 65536, 4096, 4, 128)
        for r in (1, 8, 100, 128):
            assert g.adapter_bytes(r) == lay.adapter_bytes(r) == o.adapter_bytes(r)
        assert g.adapter_bytes(0) == 0 and g.adapter_bytes(129) == 0
        pt = g.load(0, 100, 1.0)
        assert len(pt) == -(-lay.adapter_bytes(100) // 65536)
        g.close()


def test_batch_pins_adapters_and_errors_leave_pool_unchanged(oracle_mod):
    import paper_2512_20210_amd as B
    lay = Layout((64,), (64,), DT_F16)
    o, g = _pools(oracle_mod, lay, 4096, 8, 8, 16)
    g.load(0, 4, 1.0)
    g.load(5, 16, 1.0)
    before = g.stats()
    rc, _ = B.plora_batch_begin(g.h, np.array([0, 5, 3], np.int32))
    assert rc == B.PLORA_ERR_NOTFOUND
    rc, _ = B.plora_batch_begin(g.h, np.array([0, 8], np.int32))
    assert rc == B.PLORA_ERR_INVAL
    rc, _ = B.plora_batch_begin(g.h, np.array([0, -2], np.int32))
    assert rc == B.PLORA_ERR_INVAL
    assert g.stats() == before
    b1 = g.batch_begin(np.array([5, -1, 0, 5], np.int32))
    b2 = g.batch_begin(np.array([5], np.int32))
    assert B.plora_evict(g.h, 5) == B.PLORA_ERR_BUSY and B.plora_evict(g.h, 0) == B.PLORA_ERR_BUSY
    g.batch_end(b1)
    assert B.plora_evict(g.h, 0) == B.PLORA_OK
    assert B.plora_evict(g.h, 5) == B.PLORA_ERR_BUSY  # still pinned by b2
    assert B.plora_pool_destroy(g.h) == B.PLORA_ERR_BUSY
    # a placement-only pool refuses to compute
    assert B.plora_shrink(g.h, b2, 0, 1, [16], [16]) == B.PLORA_ERR_INVAL
    g.batch_end(b2)
    assert B.plora_batch_end(g.h, b2) == B.PLORA_ERR_INVAL  # already ended
    assert B.plora_evict(g.h, 5) == B.PLORA_OK
    g.close()


def test_pool_create_rejects_bad_arguments():
    import paper_2512_20210_amd as B
    ok = dict(page_bytes=4096, n_pages=4, d_in=[64], d_out=[64], dtype=B.PLORA_BF16, max_adapters=4, max_rank=16)

    def create(**kw):
        a = dict(ok, **kw)
        rc, h = B.plora_pool_create(a["page_bytes"], a["n_pages"], a["d_in"], a["d_out"], a["dtype"], a["max_adapters"],
                                    a["max_rank"], None, B.PLORA_POOL_PLACEMENT_ONLY)
        if rc == 0:
            B.plora_pool_destroy(h)
        return rc
    assert create() == B.PLORA_OK
    for bad in (dict(page_bytes=3000), dict(page_bytes=2048), dict(n_pages=0), dict(d_in=[60]), dict(d_out=[0]),
                dict(dtype=3), dict(max_adapters=0), dict(max_rank=0), dict(max_rank=513),
                dict(d_in=[1 << 20], d_out=[64]),  # 64 rows of 2 MiB over 4 KiB pages: window too large
                ):
        assert create(**bad) == B.PLORA_ERR_INVAL, bad
    assert B.plora_pool_set_option(None, "xcd_remap", 1) == B.PLORA_ERR_INVAL


def test_options_validate():
    import paper_2512_20210_amd as B
    g = B.PagedLoraPool(4096, 4, [64], [64], B.PLORA_BF16, 4, 16, placement_only=True)
    for key, good, bad in (("mfma_min_tokens", 3, -1), ("mfma_min_tokens_expand", 0, -2), ("mfma_min_work", 1, 0), ("coop_max_workgroups_shrink", 0, -1), ("batches_per_marker", 1, 0), ("staging_min_runs", 1, 0), ("panel_min_blocks", 0, -1), ("panel_half_max_workgroups", 0, -1), ("mfma_cols_max_group", 64, -1), ("mfma_shrink_depth", 2, 3), ("mfma_shrink_depth", 0, -1), ("batches_per_marker", 64, 65), ("coop_max_workgroups_expand", 5000, -1),
                           ("mfma_min_work_expand", 1000, -5), ("xcd_remap", 1, 5), ("slot_major", -1, 2), ("slot_major_expand", 2, 3), ("slot_major_shrink", 1, 2), ("xcd_remap_expand", 0, 2)):
        assert B.plora_pool_set_option(g.h, key, good) == B.PLORA_OK
        assert B.plora_pool_set_option(g.h, key, bad) == B.PLORA_ERR_INVAL
    assert B.plora_pool_set_option(g.h, "no_such_option", 1) == B.PLORA_ERR_INVAL
    assert B.plora_pool_set_option(g.h, "staging_bytes", 4096) == B.PLORA_ERR_INVAL  # a placement-only pool copies nothing
    assert B.plora_profile(g.h, 1) == B.PLORA_ERR_INVAL  # nothing to time without a device
    g.close()
