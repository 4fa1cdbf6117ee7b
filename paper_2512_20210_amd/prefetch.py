"""Proactive prefetching on top of the residency manager (Sec. III-B "Proactive Prefetching").

Before every prediction interval the caller hands over p_hat, the predicted probability that each
adapter is requested in the coming interval.  Adapters with p_hat > theta that are not in GPU memory
are loaded on the copy stream (between two decode batches, so the copies run beside the next batch's
kernels); room is made with the eviction score of Eq. 3, but never at the cost of an adapter that
is itself predicted (p_hat > theta).  p_hat also enters Eq. 3 for the on-demand evictions of the
interval.

Two sources of p_hat: the library's LSTM predictor (`LstmPredictor` in the binding: Sec. III-A,
learning online from the intervals it has seen), and `SyntheticPredictor`, which needs no learning
and so serves traces without structure to learn: it looks at the true next interval and degrades that
knowledge to a chosen quality q (the paper reports 86 % prediction accuracy; read here as q = 0.86):
every adapter that will be requested is flagged with probability q, and for every one it misses a
wrong adapter is flagged instead (drawn by popularity among those that will not be requested), so
the flagged set has the size of the true set and both recall and precision are about q.  Flagged
adapters get p_hat uniform in (theta, 1), the others uniform in (0, theta).

Counted: cold starts (requests that find their adapter not in memory and must wait for a load on
demand), useful prefetches (prefetched adapters that are requested before they are evicted) and
wasted ones.
"""
import numpy as np

from .manager import ResidencyManager


class SyntheticPredictor:
    def __init__(self, n_adapters, popularity, quality, theta=0.5, seed=0):
        assert 0.0 <= quality <= 1.0 and 0.0 < theta < 1.0
        self.n, self.q, self.theta = int(n_adapters), float(quality), float(theta)
        self.pop = np.asarray(popularity, np.float64)
        self.rng = np.random.default_rng(seed)

    def predict(self, next_interval_ids):
        """p_hat[n_adapters] for the interval whose requests are next_interval_ids."""
        need = np.unique(np.asarray(next_interval_ids, np.int64))
        keep = self.rng.random(len(need)) < self.q
        flagged = need[keep]
        n_wrong = int(len(need) - len(flagged))
        if n_wrong:
            w = self.pop.copy()
            w[need] = 0.0
            if w.sum() > 0:
                wrong = self.rng.choice(self.n, size=min(n_wrong, int((w > 0).sum())), replace=False, p=w / w.sum())
                flagged = np.concatenate([flagged, wrong])
        p_hat = self.rng.random(self.n) * self.theta
        p_hat[flagged] = self.theta + (1.0 - self.theta) * (1.0 - self.rng.random(len(flagged)))
        return p_hat


class PrefetchManager(ResidencyManager):
    def __init__(self, *args, theta=0.5, prefetch_stream=None, **kw):
        """prefetch_stream: stream of the prefetch copies; give one of its own so that a load on demand
        (on copy_stream) does not queue behind a whole interval's prefetches."""
        super().__init__(*args, **kw)
        self.theta = theta
        self.prefetch_stream = prefetch_stream
        self.prefetched = set()  # loaded by prefetch, not requested since
        self.prefetch_loads = self.useful_prefetches = self.wasted_prefetches = self.prefetch_no_room = 0

    def _on_evict(self, vid):
        if vid in self.prefetched:
            self.prefetched.discard(vid)
            self.wasted_prefetches += 1

    def begin_interval(self, p_hat):
        """Takes the prediction for the coming interval and starts the loads it asks for, most
        probable first.  Returns the ids whose load was started."""
        self.p_hat = p_hat
        want = [int(i) for i in np.argsort(-np.asarray(p_hat), kind="stable") if p_hat[i] > self.theta]
        started = []
        for aid in want:
            if aid in self.last_use:
                continue
            if not self._load(aid, may_evict=lambda i: not (self.p_hat[i] > self.theta), stream=self.prefetch_stream):
                self.prefetch_no_room += 1
                break  # no unpredicted resident left to give up its pages
            self.prefetched.add(aid)
            self.prefetch_loads += 1
            started.append(aid)
        return started

    def request(self, aid):
        was_prefetched = aid in self.prefetched
        hit = super().request(aid)
        if was_prefetched:
            self.prefetched.discard(aid)
            if hit:
                self.useful_prefetches += 1
        return hit

    @property
    def cold_starts(self):
        return self.misses
