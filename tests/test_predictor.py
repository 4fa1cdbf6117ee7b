"""The library's traffic predictor (host code, fp32) against the oracle (oracle/lstm.py, fp64).

forward + Eq. 2 : same parameters, same window -> same loss and the same p_hat;
gradient        : the library's backward pass against the oracle's central differences;
Adam            : a few updates on fixed samples against the oracle's forward / finite-difference
                  gradient / Adam chain;
history         : observe / predict / train over a replay buffer (window padding with empty intervals,
                  buffer limit, sampler range, error answers).
Tolerances: fp32 against fp64 through a few hundred sums of O(1) terms -> 2e-5 relative on losses and
probabilities; the finite-difference gradient is good to ~1e-6, the fp32 backward pass to ~1e-5 of the
largest entry.
"""
import numpy as np
import pytest

import paper_2512_20210_amd as P
from oracle import lstm as O


def _make(n, H, L, W, seed=3, **kw):
    rc, h = P.plora_predictor_create(n, window=W, hidden=H, layers=L, seed=seed, **kw)
    assert rc == P.PLORA_OK
    return h


@pytest.mark.parametrize("n,H,L,W", [(6, 4, 1, 3), (9, 5, 2, 4), (40, 16, 2, 8), (7, 3, 3, 2)])
def test_loss_and_gradient_match_the_oracle(n, H, L, W):
    h = _make(n, H, L, W)
    assert P.plora_predictor_param_count(h) == O.param_count(n, H, L)
    rng = np.random.default_rng(n + H)
    params = (rng.standard_normal(O.param_count(n, H, L)) * 0.5).astype(np.float32)
    assert P.plora_predictor_set_params(h, params) == P.PLORA_OK
    rc, back = P.plora_predictor_get_params(h)
    assert rc == P.PLORA_OK and (back == params).all()
    seq = O.feature(rng.integers(0, 4, size=(W, n)) * (rng.random((W, n)) < 0.5)).astype(np.float32)
    y = (rng.random(n) < 0.3).astype(np.float32)
    rc, loss, grad = P.plora_predictor_loss_grad(h, seq, y)
    assert rc == P.PLORA_OK
    ref = O.loss(params.astype(np.float64), seq.astype(np.float64), y, H, L)
    assert abs(loss - ref) <= 2e-5 * max(1.0, abs(ref))
    if O.param_count(n, H, L) <= 700:
        idx = list(range(O.param_count(n, H, L)))
    else:  # a sample of every block of the parameter vector
        idx = sorted(set(rng.integers(0, O.param_count(n, H, L), size=300).tolist()) | set(range(0, 40)) | set(range(O.param_count(n, H, L) - 40, O.param_count(n, H, L))))
    g_ref = O.grad_fd(params.astype(np.float64), seq.astype(np.float64), y, H, L, index=idx)
    scale = max(1.0, np.abs(g_ref).max())
    assert np.abs(grad[idx] - g_ref).max() <= 3e-5 * scale, np.abs(grad[idx] - g_ref).max()
    assert P.plora_predictor_destroy(h) == P.PLORA_OK


def test_predict_over_a_short_history_pads_with_empty_intervals():
    n, H, L, W = 8, 4, 2, 5
    h = _make(n, H, L, W)
    rc, params = P.plora_predictor_get_params(h)
    lim = 1.0 / np.sqrt(H)
    lay, w_fc, b_fc = O.unpack(params, n, H, L)
    assert np.abs(params).max() <= lim and np.abs(w_fc).max() > 0.2 * lim   # initialisation range
    assert (b_fc == 0).all() and all((b == 0).all() for _, _, b in lay)
    hist = [[1, 1, 3], [0], [2, 2, 2, 7]]
    for ids in hist:
        assert P.plora_predictor_observe(h, ids) == P.PLORA_OK
    assert P.plora_predictor_observed(h) == 3
    seq = np.zeros((W, n))
    for k, ids in enumerate(hist):
        seq[W - len(hist) + k] = O.feature(np.bincount(ids, minlength=n))
    rc, p_hat = P.plora_predictor_predict(h, n)
    ref = O.sigmoid(O.forward(params.astype(np.float64), seq, H, L))
    assert rc == P.PLORA_OK and np.abs(p_hat - ref).max() <= 2e-6


def test_adam_updates_on_fixed_samples_follow_the_oracle():
    n, H, L, W = 6, 3, 2, 3
    h = _make(n, H, L, W, replay=50, batch=2, lr=1e-2)
    rng = np.random.default_rng(12)
    hist = [rng.integers(0, n, size=rng.integers(1, 6)).tolist() for _ in range(7)]
    for ids in hist:
        assert P.plora_predictor_observe(h, ids) == P.PLORA_OK
    feats = [O.feature(np.bincount(ids, minlength=n)) for ids in hist]
    present = [(np.bincount(ids, minlength=n) > 0).astype(np.float64) for ids in hist]

    def window(end):
        s = np.zeros((W, n))
        for k in range(W):
            pos = end - W + k
            if pos >= 0:
                s[k] = feats[pos]
        return s
    rc, p0 = P.plora_predictor_get_params(h)
    p = p0.astype(np.float64)
    m, v = np.zeros_like(p), np.zeros_like(p)
    for t, batch in enumerate(([1, 4], [6, 2], [3, 3]), start=1):
        rc, loss = P.plora_predictor_train_batch(h, batch)
        assert rc == P.PLORA_OK
        g = np.zeros_like(p)
        l_ref = 0.0
        for pos in batch:
            g += O.grad_fd(p, window(pos), present[pos], H, L) / len(batch)
            l_ref += O.loss(p, window(pos), present[pos], H, L) / len(batch)
        assert abs(loss - l_ref) <= 2e-5 * max(1.0, l_ref)
        p, m, v = O.adam_step(p, m, v, g, t, lr=1e-2)
        rc, got = P.plora_predictor_get_params(h)
        # Adam divides by sqrt(v): entries whose gradient is ~0 are noise in both, compare where it is not
        big = np.abs(g) > 1e-3 * np.abs(g).max()
        assert np.abs(got[big] - p[big]).max() <= 2e-4, (t, np.abs(got[big] - p[big]).max())


def test_worker_threads_give_the_same_updates():
    n = 30
    rng = np.random.default_rng(4)
    hist = [rng.integers(0, n, size=12).tolist() for _ in range(20)]
    res = []
    for threads in (1, 3, 8):
        h = _make(n, 8, 2, 4, replay=50, batch=8, lr=1e-2)
        assert P.plora_predictor_set_threads(h, threads) == P.PLORA_OK
        for ids in hist:
            P.plora_predictor_observe(h, ids)
        rc, loss = P.plora_predictor_train(h, 6)
        assert rc == P.PLORA_OK
        res.append((loss, P.plora_predictor_get_params(h)[1]))
        P.plora_predictor_destroy(h)
    for loss, params in res[1:]:
        assert abs(loss - res[0][0]) <= 1e-4 * res[0][0]
        assert np.abs(params - res[0][1]).max() <= 5e-4      # same samples, another summation order
    h = _make(n, 8, 2, 4)
    assert P.plora_predictor_set_threads(h, 0) == P.PLORA_ERR_INVAL and P.plora_predictor_set_threads(h, 65) == P.PLORA_ERR_INVAL
    P.plora_predictor_destroy(h)


def test_replay_limit_sampler_and_errors():
    n = 5
    h = _make(n, 4, 1, 2, replay=4, batch=3)
    rc, loss = P.plora_predictor_train(h, 2)
    assert rc == P.PLORA_OK and loss == 0.0                       # nothing observed yet: no-op
    for k in range(9):
        assert P.plora_predictor_observe(h, [k % n, (2 * k) % n]) == P.PLORA_OK
    assert P.plora_predictor_observed(h) == 4                      # the oldest intervals left
    assert P.plora_predictor_observe(h, [n]) == P.PLORA_ERR_INVAL
    assert P.plora_predictor_observe(h, [-1]) == P.PLORA_ERR_INVAL
    assert P.plora_predictor_train_batch(h, [0])[0] == P.PLORA_ERR_INVAL   # position 0 has no past
    assert P.plora_predictor_train_batch(h, [4])[0] == P.PLORA_ERR_INVAL   # past the newest interval
    rc, before = P.plora_predictor_get_params(h)
    rc, loss = P.plora_predictor_train(h, 5)
    rc2, after = P.plora_predictor_get_params(h)
    assert rc == P.PLORA_OK and loss > 0 and np.isfinite(after).all() and (after != before).any()
    assert P.plora_predictor_create(0)[0] == P.PLORA_ERR_INVAL
    assert P.plora_predictor_create(4, window=0)[0] == P.PLORA_ERR_INVAL
    assert P.plora_predictor_create(4, lr=0.0)[0] == P.PLORA_ERR_INVAL
    assert P.plora_predictor_destroy(h) == P.PLORA_OK


def test_learns_a_periodic_pattern():
    """Adapters that are requested every third interval: after training, the predicted set of the next
    interval is the right third."""
    n = 12
    pr = P.LstmPredictor(n, window=6, hidden=16, layers=2, replay=200, batch=16, lr=5e-3, seed=5, train_steps=4)
    groups = [list(range(0, 4)), list(range(4, 8)), list(range(8, 12))]
    hits = total = 0
    for t in range(400):
        ids = groups[t % 3]
        p_hat = pr.predict(ids)
        if t >= 300:
            pred = set(np.nonzero(p_hat > 0.5)[0].tolist())
            hits += len(pred & set(ids)) - len(pred - set(ids))
            total += len(ids)
    pr.close()
    assert hits >= 0.9 * total, (hits, total)
