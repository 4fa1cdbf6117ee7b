"""Residency manager on top of the page pool: load on demand, evict by score.

The pool itself only places and frees pages (plora_load_adapter / plora_evict).  This module adds
the policy layer the paper describes in Sec. III-B: when memory is short, adapters are evicted by a
combined recency / frequency / prediction score (Eq. 3),

    s_i = alpha * LRU_i + beta * freq_i + gamma * p_hat_i ,

and a request for a non-resident adapter starts a host->GPU copy on the copy stream.  The paper
gives neither the weights nor the normalisation nor the direction; the reading used here: s_i is a
retention value (the lowest score is evicted), LRU_i = 1 - (rank by last use) / (n - 1) with 1 for
the most recently used, freq_i = hits in a sliding window of the last `window` requests divided by
the largest such count among resident adapters, p_hat_i supplied by the caller (the LSTM predictor's
forecast or a synthetic one), alpha = 0.4, beta = 0.3, gamma = 0.3, ties go to the lowest id.  Adapters that cannot
be evicted right now (copy still in flight, or pinned by an open batch) are skipped.

The manager is written against a minimal pool interface (load / evict / stats, raising an error
object with a .code on failure), so the same decisions can drive the CPU oracle's pool in tests.
"""
from collections import deque

import numpy as np

ERR_NOMEM, ERR_BUSY = -2, -5


class ResidencyManager:
    def __init__(self, pool, ranks, scales, blob_of, alpha=0.4, beta=0.3, gamma=0.3, window=1000, p_hat=None,
                 copy_stream=None):
        """pool: object with load(id, rank, scale, blob[, stream]) and evict(id); ranks / scales: per
        adapter id; blob_of(id) -> what the pool's load takes as the adapter's weights."""
        self.pool, self.ranks, self.scales, self.blob_of = pool, ranks, scales, blob_of
        self.alpha, self.beta, self.gamma = alpha, beta, gamma
        self.p_hat = p_hat
        self.copy_stream = copy_stream
        self.clock = 0
        self.last_use = {}            # resident id -> clock of last request
        self.recent = deque()         # sliding window of requested ids
        self.window = window
        self.count = {}               # id -> hits inside the window
        self.hits = self.misses = self.evictions = self.skipped_busy = self.failed = 0
        self.log = []                 # ("load", id) / ("evict", id) in order, for replay on another pool

    def resident(self):
        return self.last_use.keys()

    def _touch(self, aid):
        self.clock += 1
        self.recent.append(aid)
        self.count[aid] = self.count.get(aid, 0) + 1
        if len(self.recent) > self.window:
            old = self.recent.popleft()
            self.count[old] -= 1
            if not self.count[old]:
                del self.count[old]

    def scores(self):
        """Retention score of every resident adapter (Eq. 3 under the reading above)."""
        ids = sorted(self.last_use)
        n = len(ids)
        order = sorted(ids, key=lambda i: self.last_use[i])          # oldest first
        lru = {i: (k / (n - 1) if n > 1 else 1.0) for k, i in enumerate(order)}
        cmax = max([self.count.get(i, 0) for i in ids] + [1])
        out = {}
        for i in ids:
            ph = float(self.p_hat[i]) if self.p_hat is not None else 0.0
            out[i] = self.alpha * lru[i] + self.beta * self.count.get(i, 0) / cmax + self.gamma * ph
        return out

    def _on_evict(self, vid):
        """Hook for subclasses: adapter `vid` has just been evicted."""

    def _load(self, aid, may_evict=None, stream=None):
        """Loads `aid` (on `stream`, else on the manager's copy stream), evicting residents in ascending
        score order while the pool is out of pages (only those for which may_evict(id) holds, if given).
        Returns False if no room could be made."""
        victims = None
        stream = self.copy_stream if stream is None else stream
        while True:
            try:
                if stream is None:
                    self.pool.load(aid, int(self.ranks[aid]), float(self.scales[aid]), self.blob_of(aid))
                else:
                    self.pool.load(aid, int(self.ranks[aid]), float(self.scales[aid]), self.blob_of(aid), stream)
                self.log.append(("load", aid))
                self.last_use[aid] = self.clock
                return True
            except Exception as e:  # pool error object with .code
                if getattr(e, "code", None) != ERR_NOMEM:
                    raise
            if victims is None:
                sc = self.scores()
                victims = sorted((i for i in sc if may_evict is None or may_evict(i)), key=lambda i: (sc[i], i))
            evicted = False
            while victims:
                vid = victims.pop(0)
                try:
                    self.pool.evict(vid)
                except Exception as e:
                    if getattr(e, "code", None) == ERR_BUSY:
                        self.skipped_busy += 1
                        continue
                    raise
                del self.last_use[vid]
                self.log.append(("evict", vid))
                self.evictions += 1
                self._on_evict(vid)
                evicted = True
                break
            if not evicted:
                return False

    def request(self, aid):
        """Make adapter `aid` resident. Returns True on a hit, False if a load was started (or failed)."""
        self._touch(aid)
        if aid in self.last_use:
            self.last_use[aid] = self.clock
            self.hits += 1
            return True
        self.misses += 1
        if not self._load(aid):
            self.failed += 1
        return False
