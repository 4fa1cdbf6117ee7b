"""A synthetic source of access predictions (an input generator: none of the method's arithmetic).

The paper's predictor is trained on a production trace that is not available, and an i.i.d. request
trace has nothing to learn.  SyntheticPredictor stands in for a predictor of a chosen quality q: it
looks at the true next interval and degrades that knowledge: every adapter that will be requested is
flagged with probability q, and for every one it misses a wrong adapter is flagged instead (drawn by
popularity among those that will not be requested), so the flagged set has the size of the true set
and both recall and precision are about q (the paper reports 86 % prediction accuracy, read as
q = 0.86).  Flagged adapters get p_hat uniform in (theta, 1), the others uniform in (0, theta).
"""
import numpy as np


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
