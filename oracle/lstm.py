"""CPU oracle of the traffic predictor (Sec. III-A): test infrastructure, not part of the product.

Plain numpy in fp64, written from the textbook definitions so that it can be checked by eye: a
stack of LSTM layers over a window of per-interval feature vectors, a fully connected layer on the
last hidden state, the summed binary cross-entropy of Eq. 2 on its logits, and Adam.  The gradient
is taken by central differences of the loss itself (no hand-derived backward pass here: the product
has one, and this is what it is checked against).

Parameter vector (the product uses the same order so that vectors can be exchanged):
  layer 0:  E[n][4H]   input weights, one row per adapter (the learned "embedding" of the adapter;
                       gates of a step get  sum_i feature_i * E[i]),
            W_hh[4H][H], b[4H]
  layer l>0: W_ih[4H][H], W_hh[4H][H], b[4H]
  output:   W_fc[n][H], b_fc[n]
Gate order inside 4H: input, forget, cell candidate, output.
"""
import numpy as np


def feature(counts):
    """Normalised access count of one interval (Sec. III-A "we normalize counts"; the paper does not
    say how: c / (1 + c), bounded and free of global statistics, is this build's reading)."""
    c = np.asarray(counts, dtype=np.float64)
    return c / (1.0 + c)


def param_count(n, H, L):
    return n * 4 * H + 4 * H * H + 4 * H + (L - 1) * (4 * H * H + 4 * H * H + 4 * H) + n * H + n


def unpack(params, n, H, L):
    p = np.asarray(params, dtype=np.float64)
    o = 0

    def take(shape):
        nonlocal o
        k = int(np.prod(shape))
        a = p[o:o + k].reshape(shape)
        o += k
        return a
    layers = []
    for l in range(L):
        w_in = take((n, 4 * H)) if l == 0 else take((4 * H, H))
        layers.append((w_in, take((4 * H, H)), take((4 * H,))))
    w_fc, b_fc = take((n, H)), take((n,))
    assert o == p.size
    return layers, w_fc, b_fc


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def forward(params, seq, H, L):
    """seq[W][n]: feature vectors of W consecutive intervals, oldest first.  Returns the n logits."""
    seq = np.asarray(seq, dtype=np.float64)
    n = seq.shape[1]
    layers, w_fc, b_fc = unpack(params, n, H, L)
    h = [np.zeros(H) for _ in range(L)]
    c = [np.zeros(H) for _ in range(L)]
    for t in range(seq.shape[0]):
        x = seq[t]
        for l, (w_in, w_hh, b) in enumerate(layers):
            a = (x @ w_in if l == 0 else w_in @ x) + w_hh @ h[l] + b
            gi, gf, gg, go = sigmoid(a[:H]), sigmoid(a[H:2 * H]), np.tanh(a[2 * H:3 * H]), sigmoid(a[3 * H:])
            c[l] = gf * c[l] + gi * gg
            h[l] = go * np.tanh(c[l])
            x = h[l]
    return w_fc @ h[L - 1] + b_fc


def loss(params, seq, target, H, L):
    """Eq. 2 on p = sigmoid(logit): -sum_i [ y_i log p_i + (1 - y_i) log(1 - p_i) ]."""
    z = forward(params, seq, H, L)
    y = np.asarray(target, dtype=np.float64)
    # log(1 + e^z) - y z, written so that large |z| neither overflows nor loses the small term
    return float(np.sum(np.maximum(z, 0.0) + np.log1p(np.exp(-np.abs(z))) - y * z))


def grad_fd(params, seq, target, H, L, eps=1e-6, index=None):
    """Central differences of the loss in the parameters `index` (all if None)."""
    p = np.array(params, dtype=np.float64)
    idx = range(p.size) if index is None else index
    g = np.zeros(len(idx))
    for k, j in enumerate(idx):
        old = p[j]
        p[j] = old + eps
        up = loss(p, seq, target, H, L)
        p[j] = old - eps
        dn = loss(p, seq, target, H, L)
        p[j] = old
        g[k] = (up - dn) / (2 * eps)
    return g


def adam_step(p, m, v, g, t, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (t = 1 for the first): returns the new (p, m, v)."""
    m = beta1 * m + (1 - beta1) * g
    v = beta2 * v + (1 - beta2) * g * g
    mh = m / (1 - beta1 ** t)
    vh = v / (1 - beta2 ** t)
    return p - lr * mh / (np.sqrt(vh) + eps), m, v
