"""Pins for the oracle's element codecs, page counts, allocator and virtual view.

Nothing here touches a GPU.  Each check compares the oracle with something fixed outside it:
library conversions (numpy float16, torch bfloat16), the closed form ceil(S/P) and the sizes the
paper prints (Sec. II-B, Sec. III-C), allocator invariants, and a brute-force re-scan allocator.
"""
import math
import os

import numpy as np
import pytest
import torch

from workload import DT_BF16, DT_F16, DT_F32, Layout, make_adapter

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_page_counts.txt")


def test_fp16_decode_all_patterns(oracle_mod):
    from oracle.pool import decode_elt
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([decode_elt(DT_F16, int(b)) for b in bits], dtype=np.float32)
    same = (got.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(got) & np.isnan(ref))
    assert same.all()


def test_bf16_decode_all_patterns(oracle_mod):
    from oracle.pool import decode_elt
    bits = np.arange(65536, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([decode_elt(DT_BF16, int(b)) for b in bits], dtype=np.float32)
    same = (got.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(got) & np.isnan(ref))
    assert same.all()


def _encode_cases():
    rng = np.random.default_rng(7)
    vals = [rng.standard_normal(20000).astype(np.float32) * s for s in (1e-8, 1e-5, 1e-3, 1.0, 300.0, 7e4)]
    # exact ties and neighbours around half-precision and bf16 rounding boundaries
    edge = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                     2.0 ** -14, 2.0 ** -14 - 2.0 ** -26, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -8,
                     1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, 3.3895314e38, np.inf, -np.inf], dtype=np.float32)
    u = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    return np.concatenate(vals + [edge, u[np.isfinite(u)]])


def test_fp16_encode_matches_numpy(oracle_mod):
    from oracle.pool import encode_elt
    v = _encode_cases()
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).view(np.uint16)
    got = np.array([encode_elt(DT_F16, float(x)) for x in v], dtype=np.uint16)
    assert (got == ref).all()


def test_bf16_encode_matches_torch(oracle_mod):
    from oracle.pool import encode_elt
    v = _encode_cases()
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([encode_elt(DT_BF16, float(x)) for x in v], dtype=np.uint16)
    assert (got == ref).all()


def _gold_rows():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [x.strip() for x in line.split("|")]
        rows.append((f[0],) + tuple(int(x) for x in f[1:]))
    return rows


@pytest.mark.parametrize("row", _gold_rows(), ids=lambda r: r[0])
def test_page_count_golden(oracle_mod, row):
    """Adapter bytes and ceil(S/P) for the values the paper and the workloads fix."""
    name, rank, elems, elt, P, S, pages = row
    assert elt == 2
    # a single slot whose d_in + d_out equals the record's elements-per-rank
    pool = oracle_mod.OraclePool(P, pages + 3, [elems // 2], [elems - elems // 2], DT_F16, 2, rank)
    assert pool.adapter_bytes(rank) == S
    blob = np.zeros(S // 2, dtype=np.uint16)
    pt = pool.load(0, rank, 1.0, blob)
    assert len(pt) == pages == math.ceil(S / P)
    assert pool.stats()["used_pages"] == pages


def test_paper_printed_sizes():
    """Sec. II-B: rank 8 is 'roughly 13MB', rank 64 is '100MB+' on Llama2-7B."""
    rows = {r[0]: r for r in _gold_rows()}
    assert abs(rows["paper_llama7b_qkv_r8"][5] / 1e6 - 13) < 0.5
    assert 100 <= rows["paper_llama7b_qkv_r64"][5] / 1e6 < 101


def test_small_workload_uses_12_of_64_pages(oracle_mod):
    lay = Layout((1024,), (1024,), DT_F16)
    pool = oracle_mod.OraclePool(16384, 64, lay.d_in, lay.d_out, DT_F16, 4, 16)
    rng = np.random.default_rng(0)
    tables = [pool.load(i, r, 2.0, make_adapter(rng, lay, r)) for i, r in enumerate([8, 16, 8, 16])]
    assert [len(t) for t in tables] == [2, 4, 2, 4]
    # fresh pool: the k-th adapter gets the contiguous run starting at the running sum
    assert np.concatenate(tables).tolist() == list(range(12))
    st = pool.stats()
    assert st["used_pages"] == 12 and st["free_pages"] == 52


class BruteAllocator:
    """O(n^2) reference: for every page wanted, re-scan from page 0 for the first free one."""

    def __init__(self, n):
        self.free = [True] * n
        self.tables = {}

    def load(self, aid, m):
        if aid in self.tables:
            return "EXISTS"
        if sum(self.free) < m:
            return "NOMEM"
        pt = []
        for _ in range(m):
            q = 0
            while not self.free[q]:
                q += 1
            self.free[q] = False
            pt.append(q)
        self.tables[aid] = pt
        return pt

    def evict(self, aid):
        if aid not in self.tables:
            return "NOTFOUND"
        for q in self.tables.pop(aid):
            self.free[q] = True
        return "OK"


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_allocator_history_vs_bruteforce_and_invariants(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    lay = Layout((64, 32), (32, 96), DT_BF16)  # 224 elements per rank -> 448 B per rank
    P, n_pages, max_ad, max_rank = 4096, 40, 24, 128
    pool = oracle_mod.OraclePool(P, n_pages, lay.d_in, lay.d_out, DT_BF16, max_ad, max_rank)
    brute = BruteAllocator(n_pages)
    resident = {}
    for step in range(600):
        aid = int(rng.integers(0, max_ad))
        if rng.random() < 0.55:
            rank = int(rng.integers(1, max_rank + 1))
            m = math.ceil(lay.adapter_bytes(rank) / P)
            free_before = pool.stats()["free_pages"]
            exp = brute.load(aid, m)
            blob = np.full(lay.adapter_elems(rank), aid, dtype=np.uint16)
            try:
                pt = pool.load(aid, rank, 1.0, blob)
                assert isinstance(exp, list) and pt.tolist() == exp
                assert len(pt) == m
                assert (np.diff(pt) > 0).all()  # ascending
                resident[aid] = (rank, pt)
            except oracle_mod.OracleError as e:
                assert {-2: "NOMEM", -3: "EXISTS"}[e.code] == exp
                if e.code == -2:
                    # no external fragmentation: a load fails only when free pages < needed
                    assert free_before < m
                assert pool.stats()["free_pages"] == free_before  # failed call changed nothing
        else:
            exp = brute.evict(aid)
            try:
                pool.evict(aid)
                assert exp == "OK"
                resident.pop(aid)
            except oracle_mod.OracleError as e:
                assert e.code == -4 and exp == "NOTFOUND"
        # invariants after every event
        used = np.concatenate([pt for _, pt in resident.values()]) if resident else np.zeros(0, np.int32)
        assert len(np.unique(used)) == len(used)  # tables pairwise disjoint
        assert (used >= 0).all() and (used < n_pages).all()
        st = pool.stats()
        assert st["used_pages"] == len(used) and st["used_pages"] + st["free_pages"] == n_pages
        fm = pool.free_map()
        assert fm.sum() == st["free_pages"] and not fm[used].any()
        assert st["resident_bytes"] == sum(lay.adapter_bytes(r) for r, _ in resident.values())
        assert fm.tolist() == brute.free


def test_load_succeeds_iff_enough_free_pages(oracle_mod):
    """Checkerboard the pool, then ask for every free page at once: must succeed (no external
    fragmentation, Sec. III-C), and one more page must fail."""
    lay = Layout((1024,), (1024,), DT_F16)  # 4 KiB per rank
    P, n_pages = 4096, 32
    pool = oracle_mod.OraclePool(P, n_pages, lay.d_in, lay.d_out, DT_F16, 64, 32)
    for i in range(n_pages):
        pool.load(i, 1, 1.0, np.zeros(2048, np.uint16))
    for i in range(0, n_pages, 2):
        pool.evict(i)
    assert pool.stats()["free_pages"] == 16
    with pytest.raises(oracle_mod.OracleError) as ei:
        pool.load(40, 17, 1.0, np.zeros(17 * 2048, np.uint16))
    assert ei.value.code == -2
    pt = pool.load(40, 16, 1.0, np.zeros(16 * 2048, np.uint16))
    assert pt.tolist() == list(range(0, n_pages, 2))


@pytest.mark.parametrize("dtype", [DT_F16, DT_BF16, DT_F32])
def test_virtual_view_reads_back_blob(oracle_mod, dtype):
    """Scattered pages present a contiguous virtual view (Sec. III-C "Page Structure")."""
    rng = np.random.default_rng(11)
    lay = Layout((72, 40), (24, 136), dtype)
    P = 4096
    pool = oracle_mod.OraclePool(P, 64, lay.d_in, lay.d_out, dtype, 8, 40)
    blobs = {}
    for aid, rank in [(0, 5), (1, 17), (2, 40), (3, 1)]:
        blobs[aid] = make_adapter(rng, lay, rank)
        pool.load(aid, rank, 1.0, blobs[aid])
    pool.evict(1)
    blobs[4] = make_adapter(rng, lay, 33)
    pt = pool.load(4, 33, 1.0, blobs[4])
    assert (np.diff(pt) != 1).any()  # really scattered
    for aid in (0, 2, 3, 4):
        raw = blobs[aid].view(np.uint8)
        assert (pool.read_virtual(aid, 0, raw.nbytes) == raw).all()
        with pytest.raises(oracle_mod.OracleError):
            pool.read_virtual(aid, 1, raw.nbytes)


def test_error_paths(oracle_mod):
    lay = Layout((64,), (64,), DT_F16)
    pool = oracle_mod.OraclePool(4096, 4, lay.d_in, lay.d_out, DT_F16, 4, 16)
    blob = np.zeros(lay.adapter_elems(16), np.uint16)
    for bad in [dict(aid=-1, rank=4), dict(aid=4, rank=4), dict(aid=0, rank=0), dict(aid=0, rank=17)]:
        with pytest.raises(oracle_mod.OracleError) as ei:
            pool.load(bad["aid"], bad["rank"], 1.0, blob)
        assert ei.value.code == -1
    pool.load(0, 4, 1.0, blob)
    with pytest.raises(oracle_mod.OracleError) as ei:
        pool.load(0, 4, 1.0, blob)
    assert ei.value.code == -3
    with pytest.raises(oracle_mod.OracleError) as ei:
        pool.evict(1)
    assert ei.value.code == -4
    with pytest.raises(oracle_mod.OracleError):
        oracle_mod.OraclePool(3000, 4, [64], [64], DT_F16, 4, 16)  # page size not a power of two
    with pytest.raises(oracle_mod.OracleError):
        oracle_mod.OraclePool(4096, 4, [60], [64], DT_F16, 4, 16)  # d_in not a multiple of 8
