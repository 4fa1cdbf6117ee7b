"""Capacity planning on a placement-only pool: utilisation of the page pool under a request trace.

Runs the library's own allocator (PLORA_POOL_PLACEMENT_ONLY: no GPU needed) under the residency
manager and samples, after every load once the pool has first run out of pages,

    page_util = used_pages / n_pages
    byte_util = sum of resident adapter bytes / (n_pages * page_bytes)        (the stricter one)

Sec. V-D of the paper reports > 87 % memory utilisation for page-based allocation against 68 % for
a scheme that suffers from fragmentation.  For comparison `BlockPool` below is a contiguous
first-fit *block* allocator (every adapter needs one contiguous range, Sec. III-C / Fig. 2 top): it
fails with enough free bytes in total (external fragmentation), so the manager evicts more.
"""
import numpy as np

from .binding import PLORA_POOL_PLACEMENT_ONLY, PagedLoraPool  # noqa: F401
from .manager import ResidencyManager


class _Err(Exception):
    def __init__(self, code):
        super().__init__(str(code))
        self.code = code


class BlockPool:
    """Contiguous first-fit allocator over the same byte budget, in units of `granule` bytes."""

    def __init__(self, total_bytes, granule, bytes_of):
        self.n = total_bytes // granule
        self.granule, self.bytes_of = granule, bytes_of
        self.free = [(0, self.n)]  # sorted list of (start, length)
        self.where = {}
        self.nomem_with_space = self.nomem = 0

    def load(self, aid, rank, scale, blob, stream=None):
        need = -(-self.bytes_of(rank) // self.granule)
        for k, (s, ln) in enumerate(self.free):
            if ln >= need:
                if ln == need:
                    self.free.pop(k)
                else:
                    self.free[k] = (s + need, ln - need)
                self.where[aid] = (s, need)
                return np.arange(s, s + need, dtype=np.int32)
        self.nomem += 1
        if sum(ln for _, ln in self.free) >= need:
            self.nomem_with_space += 1  # external fragmentation: enough free bytes, no hole large enough
        raise _Err(-2)

    def evict(self, aid):
        s, need = self.where.pop(aid)
        self.free.append((s, need))
        self.free.sort()
        merged = []
        for st, ln in self.free:
            if merged and merged[-1][0] + merged[-1][1] == st:
                merged[-1] = (merged[-1][0], merged[-1][1] + ln)
            else:
                merged.append((st, ln))
        self.free = merged

    def used_fraction(self):
        return 1.0 - sum(ln for _, ln in self.free) / self.n


class _Sampler:
    """Wraps a pool for the manager and samples utilisation after every successful load once full."""

    def __init__(self, pool, total_bytes, bytes_of, used_bytes):
        self.pool, self.total, self.bytes_of, self.used_bytes = pool, total_bytes, bytes_of, used_bytes
        self.resident = {}
        self.filled = False
        self.byte_util, self.alloc_util = [], []

    def load(self, aid, rank, scale, blob, stream=None):
        try:
            self.pool.load(aid, rank, scale, blob)
        except Exception as e:
            if getattr(e, "code", None) == -2:
                self.filled = True
            raise
        self.resident[aid] = self.bytes_of(rank)
        if self.filled:
            self.byte_util.append(sum(self.resident.values()) / self.total)
            self.alloc_util.append(self.used_bytes() / self.total)

    def evict(self, aid):
        self.pool.evict(aid)
        del self.resident[aid]


def utilisation_under_trace(layout_d_in, layout_d_out, dtype, page_bytes, total_bytes, ranks, trace, n_events,
                            allocator="pages"):
    """Returns dict(byte_util_avg, byte_util_min, alloc_util_avg, evictions, hits, misses, failed,
    nomem_with_free_space).  allocator: "pages" (the library) or "block" (contiguous first fit)."""
    elt = 4 if dtype == 2 else 2
    per_rank = elt * (sum(layout_d_in) + sum(layout_d_out))
    bytes_of = lambda r: int(r) * per_rank  # noqa: E731
    n_pages = total_bytes // page_bytes
    if allocator == "pages":
        pool = PagedLoraPool(page_bytes, n_pages, layout_d_in, layout_d_out, dtype, len(ranks), int(max(ranks)),
                             placement_only=True)
        used = lambda: pool.stats()["used_pages"] * page_bytes  # noqa: E731
        wrapped = _Sampler(pool, n_pages * page_bytes, bytes_of, used)
    else:
        pool = BlockPool(total_bytes, 256, bytes_of)
        used = lambda: pool.used_fraction() * total_bytes  # noqa: E731
        wrapped = _Sampler(pool, total_bytes, bytes_of, used)
    mgr = ResidencyManager(wrapped, ranks, [1.0] * len(ranks), lambda i: None)
    n = 0
    for win in trace:
        for aid in win:
            mgr.request(int(aid))
            n += 1
            if n >= n_events:
                break
        if n >= n_events:
            break
    out = dict(byte_util_avg=float(np.mean(wrapped.byte_util)) if wrapped.byte_util else float("nan"),
               byte_util_min=float(np.min(wrapped.byte_util)) if wrapped.byte_util else float("nan"),
               alloc_util_avg=float(np.mean(wrapped.alloc_util)) if wrapped.alloc_util else float("nan"),
               evictions=mgr.evictions, hits=mgr.hits, misses=mgr.misses, failed=mgr.failed,
               nomem_with_free_space=getattr(pool, "nomem_with_space", 0))
    if allocator == "pages":
        pool.close()
    return out


def main():
    """Utilisation table for the churn workload (cfg3) in its two readings, by page size and allocator."""
    from workload import CONFIGS, churn_trace, draw_ranks
    cfg = CONFIGS["cfg3"]
    total = cfg["n_pages"] * cfg["page_bytes"]
    print("%-28s %-10s %-8s %9s %9s %9s %7s %7s %8s" % ("reading", "allocator", "page", "byte_avg", "byte_min", "alloc_avg",
                                                       "evict", "failed", "ext.frag"))
    for reading, n_slots, pop in (("1 layer (q,k,v,o)", 4, 4096), ("32 layers (q,k,v,o)", 128, 256)):
        d = [4096] * n_slots
        ranks = draw_ranks(np.random.default_rng(cfg["seed"]), pop, cfg["rank_choices"])
        for alloc, pages in (("pages", [16 << 10, 64 << 10, 256 << 10, 2 << 20]), ("block", [256])):
            for P in pages:
                trace = churn_trace(np.random.default_rng(cfg["seed"] + 1), cfg["n_events"], pop, cfg["zipf"], cfg["window"],
                                    cfg["burst_prob"], cfg["burst_mult"])
                r = utilisation_under_trace(d, d, cfg["dtype"], P, total, ranks, trace, cfg["n_events"], alloc)
                print("%-28s %-10s %-8s %9.4f %9.4f %9.4f %7d %7d %8d" % (
                    reading, alloc, ("%d KiB" % (P >> 10)) if P >= 1024 else "-", r["byte_util_avg"], r["byte_util_min"],
                    r["alloc_util_avg"], r["evictions"], r["failed"], r["nomem_with_free_space"]))


if __name__ == "__main__":
    main()
