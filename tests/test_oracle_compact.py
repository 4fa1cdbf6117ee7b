"""Pins for the oracle's compaction (Sec. III-C "Defragmentation").

The reading (oracle/plora_oracle.cpp, oracle_compact): resident adapters in ascending order of their
first page, each placed anew on the lowest-numbered pages among the free ones and its own, its bytes
moving with it.  Pinned by examples worked out by hand on a pool of ten pages in which an adapter of
rank r occupies exactly r pages, and by what must hold whatever the history: every adapter's bytes
read back unchanged, no page is lost or shared, no adapter moves up, tables stay ascending, the bound
on moved pages is kept, and a second call finds nothing left to do.
"""
import numpy as np
import pytest

from workload import DT_BF16, Layout, make_adapter

# one slot 1024 -> 1024 in 2-byte elements: 4096 bytes per unit of rank = one 4 KiB page
LAY = Layout((1024,), (1024,), DT_BF16)
PAGE = 4096


def _pool(oracle_mod, n_pages=10, max_adapters=8, max_rank=8):
    return oracle_mod.OraclePool(PAGE, n_pages, LAY.d_in, LAY.d_out, LAY.dtype, max_adapters, max_rank)


def _blob(i, rank):
    return make_adapter(np.random.default_rng(100 + i), LAY, rank)


def _example(oracle_mod):
    """a1 = {1,2,3,4}, a5 = {5,9}, a3 = {6,7,8}, page 0 free."""
    p = _pool(oracle_mod)
    blobs = {}
    for i, r in ((0, 1), (1, 4), (2, 1), (3, 3), (4, 1)):
        blobs[i] = _blob(i, r)
        p.load(i, r, 1.0, blobs[i])
    p.evict(2)
    p.evict(4)
    blobs[5] = _blob(5, 2)
    assert p.load(5, 2, 1.0, blobs[5]).tolist() == [5, 9]
    p.evict(0)
    assert p.page_table(1).tolist() == [1, 2, 3, 4] and p.page_table(3).tolist() == [6, 7, 8]
    assert np.flatnonzero(p.free_map()).tolist() == [0]
    return p, blobs


def _bytes_intact(p, blobs, ids):
    for i in ids:
        raw = np.ascontiguousarray(blobs[i]).view(np.uint8).ravel()
        assert (p.read_virtual(i, 0, len(raw)) == raw).all(), "adapter %d reads back differently" % i


def test_hand_worked_slide(oracle_mod):
    p, blobs = _example(oracle_mod)
    # a1 (first page 1) takes {0,1,2,3}: 4 pages change, page 4 is free; a5 (first page 5) takes the lowest
    # two of {4} + {5,9} = {4,5}: 2 change, page 9 is free; a3 keeps {6,7,8}: lower pages are all taken
    assert p.compact() == (6, 2)
    assert p.page_table(1).tolist() == [0, 1, 2, 3]
    assert p.page_table(5).tolist() == [4, 5]
    assert p.page_table(3).tolist() == [6, 7, 8]
    assert np.flatnonzero(p.free_map()).tolist() == [9]
    _bytes_intact(p, blobs, (1, 3, 5))
    assert p.compact() == (0, 0)
    p.close()


def test_hand_worked_bound_on_moved_pages(oracle_mod):
    p, blobs = _example(oracle_mod)
    assert p.compact(max_pages=3) == (0, 0)  # a1 needs 4: nothing moves, and the call ends there
    assert p.page_table(1).tolist() == [1, 2, 3, 4] and p.page_table(5).tolist() == [5, 9]
    assert p.compact(max_pages=4) == (4, 1)  # a1 fits; a5 would need 2 more
    assert p.page_table(1).tolist() == [0, 1, 2, 3] and p.page_table(5).tolist() == [5, 9]
    assert np.flatnonzero(p.free_map()).tolist() == [4]
    assert p.compact(max_pages=2) == (2, 1)
    assert p.page_table(5).tolist() == [4, 5]
    _bytes_intact(p, blobs, (1, 3, 5))
    p.close()


def test_hand_worked_skipped_adapter_stays(oracle_mod):
    p, blobs = _example(oracle_mod)
    # without a1: a5 takes the lowest two of {0} + {5,9} = {0,5} (both of its logical pages change place:
    # 5 -> 0 and 9 -> 5), a3 finds only page 9 free
    assert p.compact(skip=[1]) == (2, 1)
    assert p.page_table(1).tolist() == [1, 2, 3, 4]
    assert p.page_table(5).tolist() == [0, 5]
    assert p.page_table(3).tolist() == [6, 7, 8]
    assert np.flatnonzero(p.free_map()).tolist() == [9]
    _bytes_intact(p, blobs, (1, 3, 5))
    p.close()


def test_hand_worked_nothing_to_gain(oracle_mod):
    """x = {0,5} around y = {1,2,3,4}: no lower page is free for either, so both stay (x stays split)."""
    p = _pool(oracle_mod)
    blobs = {i: _blob(i, r) for i, r in ((0, 1), (1, 4), (2, 1), (3, 2))}
    for i in (0, 1, 2):
        p.load(i, (1, 4, 1)[i], 1.0, blobs[i])
    p.evict(0)
    p.evict(2)
    assert p.load(3, 2, 1.0, blobs[3]).tolist() == [0, 5]
    assert p.compact() == (0, 0)
    assert p.page_table(3).tolist() == [0, 5] and p.page_table(1).tolist() == [1, 2, 3, 4]
    p.close()


def test_empty_pool_and_bad_arguments(oracle_mod):
    p = _pool(oracle_mod)
    assert p.compact() == (0, 0)
    assert p.compact(max_pages=5, skip=[0, 3]) == (0, 0)
    p.close()


@pytest.mark.parametrize("seed", range(8))
def test_invariants_over_random_histories(oracle_mod, seed):
    rng = np.random.default_rng(500 + seed)
    n_pages, n_ad = 64, 24
    p = oracle_mod.OraclePool(PAGE, n_pages, LAY.d_in, LAY.d_out, LAY.dtype, n_ad, 8)
    blobs, ranks = {}, {}
    for step in range(300):
        i = int(rng.integers(0, n_ad))
        if i in blobs:
            p.evict(i)
            del blobs[i], ranks[i]
        else:
            r = int(rng.integers(1, 9))
            b = _blob(1000 * seed + step, r)
            try:
                p.load(i, r, 1.0, b)
            except oracle_mod.OracleError as e:
                assert e.code == -2
                continue
            blobs[i], ranks[i] = b, r
        if step % 7 == 6:
            before = {k: p.page_table(k).tolist() for k in blobs}
            free_before = p.free_map()
            bound = int(rng.choice([0, 0, 1, 5, 20]))
            skip = [k for k in blobs if rng.random() < 0.2]
            pages, adapters = p.compact(max_pages=bound, skip=skip)
            after = {k: p.page_table(k).tolist() for k in blobs}
            assert bound == 0 or pages <= bound
            assert pages == sum(x != y for k in blobs for x, y in zip(before[k], after[k]))
            assert adapters == sum(before[k] != after[k] for k in blobs)
            used = [q for k in blobs for q in after[k]]
            assert len(used) == len(set(used)), "a page belongs to two adapters"
            free_after = p.free_map()
            assert sorted(used + np.flatnonzero(free_after).tolist()) == list(range(n_pages))
            assert free_after.sum() == free_before.sum()
            for k in blobs:
                assert len(after[k]) == ranks[k] and after[k] == sorted(after[k])
                assert all(x <= y for x, y in zip(after[k], before[k])), "an adapter moved up"
                if k in skip:
                    assert after[k] == before[k]
            _bytes_intact(p, blobs, blobs.keys())
            if bound == 0:
                assert p.compact(skip=skip) == (0, 0)  # nothing left to gain
                if not skip and len(free_after) and free_after.any():
                    # with every adapter taking part, the lowest free page can only have gone up
                    assert np.flatnonzero(free_after)[0] >= np.flatnonzero(free_before)[0]
    p.close()
