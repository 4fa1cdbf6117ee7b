"""CPU oracle of the residency policy (TEST INFRASTRUCTURE ONLY; shares nothing with the library).

Sec. III-B of the paper: adapters are loaded on demand; when GPU memory is short, residents are evicted
by a combined recency / frequency / prediction score (Eq. 3),

    s_i = alpha * LRU_i + beta * freq_i + gamma * p_hat_i ,

and ("Proactive Prefetching") adapters whose predicted access probability exceeds a threshold theta
are loaded ahead of their requests.  The paper fixes neither the weights, nor how the three terms are
normalised, nor which end of the score is evicted, nor theta.  The reading written out here, step by
step, in plain Python floats (IEEE double, one rounding per operation):

  * s_i is a retention value: the LOWEST score is evicted first; equal scores go by lowest id.
  * The clock counts requests.  LRU_i: order the n residents by the clock value of their last request,
    oldest first, equal clocks by id; the adapter at position k gets k / (n - 1), a lone resident 1.
  * freq_i: requests for i among the last `window` requests, divided by the largest such count over the
    residents (never less than 1).
  * p_hat_i: the latest prediction handed over, 0 before the first.
  * s_i = ((alpha * LRU_i) + (beta * freq_i)) + (gamma * p_hat_i).
  * A load that finds the pool full scores the residents once and evicts in that order until it fits.
  * Prefetch round: candidates are the adapters with p_hat > theta, most probable first (equal
    probabilities by id); residents are skipped; room is made only among residents with p_hat <= theta;
    when none is left the round ends.  A loaded adapter starts with last use = the current clock.

Pins (tests/test_oracle_manager.py): hand-worked examples with three and four adapters for each term on
its own and combined, the tie rule, the never-evict-a-predicted-adapter rule, and the bookkeeping
identities of the counters.  No library result is ever an expected value there.
"""
from collections import Counter, deque

NOMEM = -2


class OracleManager:
    def __init__(self, pool, n_adapters, alpha=0.4, beta=0.3, gamma=0.3, theta=0.5, window=1000):
        """pool: an oracle.OraclePool (its load raises OracleError with .code == -2 when pages run out)."""
        self.pool = pool
        self.n = int(n_adapters)
        self.alpha, self.beta, self.gamma, self.theta, self.window = float(alpha), float(beta), float(gamma), float(theta), int(window)
        self.rank = [0] * self.n
        self.scale = [0.0] * self.n
        self.blob = [None] * self.n
        self.p_hat = None
        self.clock = 0
        self.recent = deque()
        self.last_use = {}          # resident id -> clock value of its last request (or of its load)
        self.prefetched = set()     # prefetched and not requested since
        self.log = []               # (0, id) = load, (1, id) = evict, in order
        self.hits = self.misses = self.loads = self.evictions = self.failed_loads = 0
        self.prefetch_loads = self.useful_prefetches = self.wasted_prefetches = self.prefetch_no_room = 0
        self.filled = False
        self.page_util, self.byte_util = [], []

    def set_adapter(self, aid, rank, scale, blob):
        self.rank[aid], self.scale[aid], self.blob[aid] = int(rank), float(scale), blob

    def residents(self):
        return sorted(self.last_use)

    def scores(self):
        """{resident id: s_i} (Eq. 3 under the reading in the module text)."""
        ids = sorted(self.last_use)
        n = len(ids)
        by_use = sorted(ids, key=lambda i: (self.last_use[i], i))
        position = {i: k for k, i in enumerate(by_use)}
        in_window = Counter(self.recent)             # requests per adapter among the last `window` requests
        counts = {i: in_window[i] for i in ids}
        cmax = max([1] + list(counts.values()))
        out = {}
        for i in ids:
            lru = position[i] / (n - 1) if n > 1 else 1.0
            freq = counts[i] / cmax
            p = float(self.p_hat[i]) if self.p_hat is not None else 0.0
            out[i] = ((self.alpha * lru) + (self.beta * freq)) + (self.gamma * p)
        return out

    def _predicted(self, aid):
        return self.p_hat is not None and float(self.p_hat[aid]) > self.theta

    def _try_load(self, aid):
        try:
            self.pool.load(aid, self.rank[aid], self.scale[aid], self.blob[aid])
        except Exception as e:
            if getattr(e, "code", None) == NOMEM:
                return False
            raise
        return True

    def _load(self, aid, spare_predicted):
        victims = None
        while not self._try_load(aid):
            self.filled = True
            if victims is None:
                sc = self.scores()
                victims = sorted((i for i in sc if not (spare_predicted and self._predicted(i))), key=lambda i: (sc[i], i))
            if not victims:
                return False
            v = victims.pop(0)
            self.pool.evict(v)
            del self.last_use[v]
            self.log.append((1, v))
            self.evictions += 1
            if v in self.prefetched:
                self.prefetched.discard(v)
                self.wasted_prefetches += 1
        self.last_use[aid] = self.clock
        self.log.append((0, aid))
        self.loads += 1
        if self.filled:
            st = self.pool.stats()
            self.page_util.append(st["used_pages"] / st["n_pages"])
            self.byte_util.append(st["resident_bytes"] / (st["n_pages"] * st["page_bytes"]))
        return True

    def request(self, aid):
        """True on a hit; False when the adapter was not resident (its load is started, or fails)."""
        self.clock += 1
        self.recent.append(aid)
        if len(self.recent) > self.window:
            self.recent.popleft()
        was_prefetched = aid in self.prefetched
        self.prefetched.discard(aid)
        if aid in self.last_use:
            self.last_use[aid] = self.clock
            self.hits += 1
            if was_prefetched:
                self.useful_prefetches += 1
            return True
        self.misses += 1
        if not self._load(aid, spare_predicted=False):
            self.failed_loads += 1
        return False

    def prefetch(self, p_hat):
        """Takes the prediction of the coming interval; returns the ids whose load was started."""
        self.p_hat = p_hat
        want = [i for i in range(self.n) if self._predicted(i)]
        want.sort(key=lambda i: (-float(p_hat[i]), i))
        started = []
        for aid in want:
            if aid in self.last_use or self.rank[aid] == 0:
                continue
            if not self._load(aid, spare_predicted=True):
                self.prefetch_no_room += 1
                break
            self.prefetched.add(aid)
            self.prefetch_loads += 1
            started.append(aid)
        return started
