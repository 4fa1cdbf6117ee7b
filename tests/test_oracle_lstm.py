"""Pins of the predictor oracle (oracle/lstm.py, Sec. III-A) against library routines and closed forms.

forward   : torch.nn.LSTM + torch.nn.Linear in fp64 with the same weights (a library routine);
loss      : torch's binary_cross_entropy_with_logits(reduction="sum") and the closed form at logit 0;
gradient  : the oracle's central differences against torch autograd through the library modules;
Adam      : torch.optim.Adam over several steps; the first step has the closed form -lr * sign(g).
A transposed weight, a swapped gate, a dropped bias, a wrong sign in Eq. 2 or a missing bias
correction in Adam fails at least one of them.
"""
import numpy as np
import pytest

from oracle import lstm as O

torch = pytest.importorskip("torch")


def _torch_model(params, n, H, L):
    layers, w_fc, b_fc = O.unpack(params, n, H, L)
    m = torch.nn.LSTM(n, H, num_layers=L).double()
    fc = torch.nn.Linear(H, n).double()
    with torch.no_grad():
        for l, (w_in, w_hh, b) in enumerate(layers):
            w_ih = w_in.T if l == 0 else w_in          # layer 0 is stored adapter-major (n x 4H)
            getattr(m, "weight_ih_l%d" % l).copy_(torch.from_numpy(np.ascontiguousarray(w_ih)))
            getattr(m, "weight_hh_l%d" % l).copy_(torch.from_numpy(w_hh))
            getattr(m, "bias_ih_l%d" % l).copy_(torch.from_numpy(b))
            getattr(m, "bias_hh_l%d" % l).zero_()
        fc.weight.copy_(torch.from_numpy(w_fc))
        fc.bias.copy_(torch.from_numpy(b_fc))
    return m, fc


@pytest.mark.parametrize("n,H,L,W", [(5, 3, 1, 4), (7, 4, 2, 6), (12, 8, 3, 3)])
def test_forward_and_loss_equal_the_library_lstm(n, H, L, W):
    rng = np.random.default_rng(n * 100 + H)
    params = rng.standard_normal(O.param_count(n, H, L)) * 0.4
    seq = O.feature(rng.integers(0, 4, size=(W, n)))
    y = (rng.random(n) < 0.3).astype(np.float64)
    m, fc = _torch_model(params, n, H, L)
    out, _ = m(torch.from_numpy(seq).unsqueeze(1))
    z_ref = fc(out[-1, 0]).detach().numpy()
    z = O.forward(params, seq, H, L)
    assert np.abs(z - z_ref).max() < 1e-12
    l_ref = torch.nn.functional.binary_cross_entropy_with_logits(torch.from_numpy(z_ref), torch.from_numpy(y), reduction="sum")
    assert abs(O.loss(params, seq, y, H, L) - float(l_ref)) < 1e-10


def test_loss_closed_forms():
    n, H, L = 6, 2, 1
    params = np.zeros(O.param_count(n, H, L))          # all logits 0: p = 1/2 whatever the target
    seq = O.feature(np.ones((3, n)))
    assert abs(O.loss(params, seq, np.zeros(n), H, L) - n * np.log(2.0)) < 1e-14
    assert abs(O.loss(params, seq, np.ones(n), H, L) - n * np.log(2.0)) < 1e-14
    params[-n:] = 30.0                                  # confident "accessed": ~0 if right, ~30 per adapter if wrong
    assert O.loss(params, seq, np.ones(n), H, L) < 1e-10
    assert abs(O.loss(params, seq, np.zeros(n), H, L) - 30.0 * n) < 1e-9


def test_feature_normalisation():
    assert O.feature([0, 1, 3]).tolist() == [0.0, 0.5, 0.75]


def test_finite_difference_gradient_equals_autograd():
    n, H, L, W = 6, 3, 2, 4
    rng = np.random.default_rng(7)
    params = rng.standard_normal(O.param_count(n, H, L)) * 0.5
    seq = O.feature(rng.integers(0, 3, size=(W, n)))
    y = (rng.random(n) < 0.4).astype(np.float64)
    m, fc = _torch_model(params, n, H, L)
    out, _ = m(torch.from_numpy(seq).unsqueeze(1))
    l = torch.nn.functional.binary_cross_entropy_with_logits(fc(out[-1, 0]), torch.from_numpy(y), reduction="sum")
    l.backward()
    layers, _, _ = O.unpack(params, n, H, L)
    ref = []
    for k in range(L):
        g_ih = getattr(m, "weight_ih_l%d" % k).grad.numpy()
        ref += [(g_ih.T if k == 0 else g_ih).reshape(-1), getattr(m, "weight_hh_l%d" % k).grad.numpy().reshape(-1),
                getattr(m, "bias_ih_l%d" % k).grad.numpy()]
    ref += [fc.weight.grad.numpy().reshape(-1), fc.bias.grad.numpy()]
    ref = np.concatenate(ref)
    g = O.grad_fd(params, seq, y, H, L)
    assert np.abs(g - ref).max() < 1e-6 * max(1.0, np.abs(ref).max())


def test_adam_equals_the_library_optimizer():
    rng = np.random.default_rng(3)
    p0 = rng.standard_normal(9)
    grads = rng.standard_normal((6, 9))
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    p, m, v = p0.copy(), np.zeros(9), np.zeros(9)
    for t in range(6):
        tp.grad = torch.from_numpy(grads[t].copy())
        opt.step()
        p, m, v = O.adam_step(p, m, v, grads[t], t + 1)
        assert np.abs(p - tp.detach().numpy()).max() < 1e-14
    # first step: m_hat / sqrt(v_hat) = g / |g|
    p1, _, _ = O.adam_step(p0, np.zeros(9), np.zeros(9), grads[0], 1)
    assert np.abs((p1 - p0) + 1e-3 * np.sign(grads[0])).max() < 1e-9
