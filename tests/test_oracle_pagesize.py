"""Pins of the page-size oracle (oracle/pagesize.py) and the library's plora_suggest_page_bytes against it.

Hand-worked expected values (the arithmetic is in the comments) and the adapter sizes the paper prints in
Sec. II-B (rank 8 = 13 MB, rank 64 = 100 MB+ for a 7B model: 32 layers x q,k,v 4096 -> 4096 at 2 bytes), for which
the paper's default page of 2 MB wastes nothing.  No library result is an expected value of the oracle's.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle.pagesize import adapter_bytes, frag, suggest_page_bytes


def test_hand_worked_fragmentation():
    # one slot 64 -> 64 at 2 bytes: S(r) = 256 r.  rank 16 = 4096 B, rank 24 = 6144 B
    assert adapter_bytes([64], [64], 2, 16) == 4096 and adapter_bytes([64], [64], 2, 24) == 6144
    assert frag(4096, [4096], [1]) == 0                         # fits exactly
    assert frag(8192, [4096], [1]) == Fraction(1, 2)            # one page, half empty
    assert frag(4096, [6144], [1]) == Fraction(2048, 8192)      # two pages, the second half empty
    # equal shares of both ranks at 4 KiB pages: (0 + 2048) wasted of (4096 + 8192) held
    assert frag(4096, [4096, 6144], [1, 1]) == Fraction(2048, 12288)
    # three times as many rank-16 adapters: (0 + 2048) of (3 * 4096 + 8192)
    assert frag(4096, [4096, 6144], [3, 1]) == Fraction(2048, 20480)


def test_hand_worked_choice():
    # ranks 16 and 32 (4096 and 8192 B): 4 KiB pages waste nothing, 8 KiB pages waste 4096 of 16384 = 25 %
    assert suggest_page_bytes([64], [64], 2, [16, 32], [1, 1], bound=0.02, max_page=65536) == (4096, 0)
    assert suggest_page_bytes([64], [64], 2, [16, 32], [1, 1], bound=0.25, max_page=65536) == (8192, Fraction(1, 4))
    # 16 KiB: (12288 + 8192) of 32768 = 62.5 %: a bound of 0.7 admits it; 32 KiB, (28672 + 24576) of 65536 = 81 %, not
    assert suggest_page_bytes([64], [64], 2, [16, 32], [1, 1], bound=0.7, max_page=65536) == (16384, Fraction(5, 8))
    # nothing meets a bound of 0 once the smallest page is 8 KiB: the least wasteful candidate, 8 KiB
    assert suggest_page_bytes([64], [64], 2, [16, 32], [1, 1], bound=0.0, min_page=8192, max_page=65536) == (8192, Fraction(1, 4))
    # a tie between candidates goes to the smaller page: rank 64 = 16 KiB wastes nothing at 4, 8 and 16 KiB
    assert suggest_page_bytes([64], [64], 2, [64], [1], bound=0.0, max_page=16384) == (16384, 0)


def test_the_papers_printed_sizes_fit_its_default_page_exactly():
    d = [4096] * 96                                             # 32 layers x q, k, v
    s8, s64 = adapter_bytes(d, d, 2, 8), adapter_bytes(d, d, 2, 64)
    assert (s8, s64) == (12582912, 100663296)                   # 12.58 MB and 100.7 MB (Sec. II-B: 13 MB, 100 MB+)
    assert s8 == 6 * (2 << 20) and s64 == 48 * (2 << 20)
    assert suggest_page_bytes(d, d, 2, [8, 16, 32, 64], [1, 1, 1, 1], bound=0.0, max_page=2 << 20) == (2 << 20, 0)
    # rank 4 is three pages exactly; rank 1 (1.5 MiB) leaves a quarter of its one page empty
    assert adapter_bytes(d, d, 2, 4) == 3 * (2 << 20)
    assert adapter_bytes(d, d, 2, 1) == 1572864 and frag(2 << 20, [1572864], [1]) == Fraction(524288, 2097152)


@pytest.mark.parametrize("seed", range(6))
def test_library_choice_equals_the_oracles(seed):
    import paper_2512_20210_amd as P
    rng = np.random.default_rng(seed)
    n_slots = int(rng.integers(1, 7))
    d_in = (8 * rng.integers(1, 600, size=n_slots)).tolist()
    d_out = (8 * rng.integers(1, 600, size=n_slots)).tolist()
    dtype = int(rng.integers(0, 3))
    elt = 4 if dtype == 2 else 2
    ranks = rng.integers(1, 129, size=int(rng.integers(1, 9))).tolist()
    weights = [k / 8 for k in rng.integers(0, 33, size=len(ranks)).tolist()]   # eighths: exact in double
    if sum(weights) == 0:
        weights[0] = 1.0
    for bound in (0.0, 0.01, 0.02, 0.1, 0.5):
        for lo, hi in ((4096, 2 << 20), (65536, 65536), (16384, 1 << 20)):
            rc, page, fr = P.plora_suggest_page_bytes(d_in, d_out, dtype, ranks, weights, bound, lo, hi)
            want_page, want_frag = suggest_page_bytes(d_in, d_out, elt, ranks, weights, bound, lo, hi)
            assert rc == P.PLORA_OK
            # a frag within a rounding of the bound could fall either way in double arithmetic: such cases are skipped
            near = any(abs(float(frag(p, [adapter_bytes(d_in, d_out, elt, r) for r in ranks], weights)) - bound) < 1e-12
                       for p in (lo << k for k in range(12)) if p <= hi)
            if not near:
                assert page == want_page, (seed, bound, lo, hi)
                assert abs(fr - float(want_frag)) < 1e-12


def test_library_argument_checks():
    import paper_2512_20210_amd as P
    ok = dict(d_in=[64], d_out=[64], dtype=1, ranks=[8], weights=[1.0])
    assert P.plora_suggest_page_bytes(**ok)[0] == P.PLORA_OK
    for bad in (dict(ranks=[0]), dict(weights=[-1.0]), dict(weights=[0.0]), dict(max_internal_frag=1.0), dict(max_internal_frag=-0.1),
                dict(min_page=2048), dict(min_page=12288), dict(min_page=1 << 20, max_page=65536), dict(ranks=[], weights=[])):
        assert P.plora_suggest_page_bytes(**dict(ok, **bad))[0] == P.PLORA_ERR_INVAL, bad
