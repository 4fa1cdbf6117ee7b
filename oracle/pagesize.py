"""CPU oracle of the page-size choice (TEST INFRASTRUCTURE ONLY; shares nothing with the library).

The paper's discussion section names adaptive page sizes "based on workload characteristics" as future
work and gives no rule; Sec. III-C fixes only that an adapter of S bytes occupies ceil(S / P) pages.  The
reading written out here: for every power of two P in [min_page, max_page] the expected internal
fragmentation of the workload's adapters is

    frag(P) = sum_k w_k (ceil(S_k / P) P - S_k) / sum_k w_k ceil(S_k / P) P ,

and the choice is the largest P with frag(P) <= bound; if none meets it, the P with the least frag (the
smaller P on a tie).  Exact rational arithmetic (fractions), so that the comparison with the bound has no
rounding of its own.

Pins (tests/test_oracle_pagesize.py): hand-worked cases, and the adapter sizes the paper prints in Sec. II-B.
"""
from fractions import Fraction


def adapter_bytes(d_in, d_out, elt, rank):
    return rank * elt * (sum(d_in) + sum(d_out))


def frag(page, sizes, weights):
    wasted = sum(Fraction(w) * (-(-s // page) * page - s) for s, w in zip(sizes, weights))
    held = sum(Fraction(w) * (-(-s // page) * page) for s, w in zip(sizes, weights))
    return wasted / held


def suggest_page_bytes(d_in, d_out, elt, ranks, weights, bound=0.02, min_page=4096, max_page=2 << 20):
    """-> (page bytes, its frag as a Fraction)."""
    sizes = [adapter_bytes(d_in, d_out, elt, r) for r in ranks]
    pages = []
    p = min_page
    while p <= max_page:
        pages.append(p)
        p *= 2
    table = [(p, frag(p, sizes, weights)) for p in pages]
    ok = [(p, f) for p, f in table if f <= Fraction(bound)]
    if ok:
        return ok[-1]
    return min(table, key=lambda pf: (pf[1], pf[0]))
