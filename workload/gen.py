"""Input generators: element codecs for storage, adapter blobs, activations, assignments."""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

DT_F16, DT_BF16, DT_F32 = 0, 1, 2
ELT_BYTES = {DT_F16: 2, DT_BF16: 2, DT_F32: 4}
RAW_DTYPE = {DT_F16: np.uint16, DT_BF16: np.uint16, DT_F32: np.float32}

__all__ = ["DT_F16", "DT_BF16", "DT_F32", "ELT_BYTES", "RAW_DTYPE", "to_elt", "from_elt", "Layout",
           "make_adapter", "make_adapters", "slot_views", "zipf_probs", "draw_tok2adapter", "make_act",
           "prefill_requests", "churn_trace", "periodic_trace", "draw_ranks"]


def to_elt(a, dtype):
    """float array -> raw storage array (uint16 bit patterns for fp16/bf16, float32)."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == DT_F32:
        return np.ascontiguousarray(a)
    if dtype == DT_F16:
        return np.ascontiguousarray(a.astype(np.float16)).view(np.uint16)
    u = np.ascontiguousarray(a).view(np.uint32)
    return ((u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)).astype(np.uint16)


def from_elt(raw, dtype):
    """raw storage array -> float32 values."""
    raw = np.asarray(raw)
    if dtype == DT_F32:
        return raw.astype(np.float32, copy=False)
    if dtype == DT_F16:
        return raw.view(np.float16).astype(np.float32)
    return (raw.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Layout:
    """The slots (linear maps d_in -> d_out) every adapter of a pool covers, and the element type."""
    d_in: tuple
    d_out: tuple
    dtype: int

    @property
    def n_slots(self):
        return len(self.d_in)

    @property
    def elt(self):
        return ELT_BYTES[self.dtype]

    @property
    def elems_per_rank(self):
        return int(sum(self.d_in) + sum(self.d_out))

    def adapter_elems(self, rank):
        return rank * self.elems_per_rank

    def adapter_bytes(self, rank):
        return self.adapter_elems(rank) * self.elt

    def slot_elem_offsets(self, slot, rank):
        """(first element of A_slot, first element of B_slot) inside a rank-`rank` blob."""
        before = sum(self.d_in[:slot]) + sum(self.d_out[:slot])
        a0 = rank * before
        return a0, a0 + rank * self.d_in[slot]


def slot_views(layout, rank, blob):
    """Per slot: (A raw view (rank, d_in), B raw view (rank, d_out)) into a packed blob."""
    out = []
    for s in range(layout.n_slots):
        a0, b0 = layout.slot_elem_offsets(s, rank)
        A = blob[a0:a0 + rank * layout.d_in[s]].reshape(rank, layout.d_in[s])
        B = blob[b0:b0 + rank * layout.d_out[s]].reshape(rank, layout.d_out[s])
        out.append((A, B))
    return out


def make_adapter(rng, layout, rank, out=None):
    """One adapter blob, slot after slot as [A_s | B_s]: A_s ~ N(0, 1/d_in) (variance), B_s ~ N(0, 1/rank)."""
    n = layout.adapter_elems(rank)
    blob = out if out is not None else np.empty(n, dtype=RAW_DTYPE[layout.dtype])
    assert blob.shape == (n,)
    for s in range(layout.n_slots):
        a0, b0 = layout.slot_elem_offsets(s, rank)
        na, nb = rank * layout.d_in[s], rank * layout.d_out[s]
        a = rng.standard_normal(na, dtype=np.float32) * np.float32(layout.d_in[s] ** -0.5)
        blob[a0:a0 + na] = to_elt(a, layout.dtype)
        b = rng.standard_normal(nb, dtype=np.float32) * np.float32(rank ** -0.5)
        blob[b0:b0 + nb] = to_elt(b, layout.dtype)
    return blob


def make_adapters(seed, layout, ranks, outs=None, workers=1):
    """Blobs for adapters 0..len(ranks)-1, adapter i drawn from its own child stream of `seed`."""
    children = np.random.SeedSequence(seed).spawn(len(ranks))

    def one(i):
        return make_adapter(np.random.default_rng(children[i]), layout, int(ranks[i]),
                            None if outs is None else outs[i])
    if workers <= 1:
        return [one(i) for i in range(len(ranks))]
    with ThreadPoolExecutor(workers) as ex:
        return list(ex.map(one, range(len(ranks))))


def draw_ranks(rng, n, choices):
    return rng.choice(np.asarray(choices, dtype=np.int32), size=n).astype(np.int32)


def zipf_probs(n, s):
    """p_i proportional to (i+1)^-s over ids 0..n-1 (id 0 is the hottest)."""
    w = (np.arange(n, dtype=np.float64) + 1.0) ** (-float(s))
    return w / w.sum()


def draw_tok2adapter(rng, T, ids, s=None, none_frac=0.0):
    """Token -> adapter id: Zipf(s) over the order of `ids` (uniform if s is None); a fraction
    none_frac of tokens gets -1 (no adapter)."""
    ids = np.asarray(ids, dtype=np.int32)
    p = None if s is None else zipf_probs(len(ids), s)
    t2a = ids[rng.choice(len(ids), size=T, p=p)].astype(np.int32)
    if none_frac > 0:
        t2a[rng.random(T) < none_frac] = -1
    return t2a


def make_act(rng, T, d, dtype, std=1.0):
    """Activations ~ N(0, std^2) as a raw (T, d) array."""
    return to_elt(rng.standard_normal((T, d), dtype=np.float32) * np.float32(std), dtype)


def prefill_requests(rng, n_requests, len_lo, len_hi, ids, s):
    """Prefill batch: request lengths uniform in [len_lo, len_hi], one Zipf(s) adapter per request.
    Returns (tok2adapter over the concatenated tokens, lengths, request adapters)."""
    lens = rng.integers(len_lo, len_hi + 1, size=n_requests)
    req = draw_tok2adapter(rng, n_requests, ids, s)
    return np.repeat(req, lens).astype(np.int32), lens, req


def churn_trace(rng, n_events, population, s, window=100, burst_prob=0.1, burst_mult=8):
    """Adapter-request trace with Zipf(s) popularity and bursts: the trace is cut into windows
    of `window` base-rate requests; each window is a burst with probability burst_prob and then
    carries burst_mult times as many requests.  Returns a list of int32 arrays, one per window,
    whose total length is at least n_events (the caller stops after n_events)."""
    p = zipf_probs(population, s)
    out, total = [], 0
    while total < n_events:
        k = window * (burst_mult if rng.random() < burst_prob else 1)
        out.append(rng.choice(population, size=k, p=p).astype(np.int32))
        total += k
    return out


def periodic_trace(rng, n_windows, population, s, window=100, n_periodic=300, periods=(2, 3, 4, 6, 8, 12)):
    """Adapter-request trace with a recurring part (the stand-in for the timer-driven functions of a
    production serverless trace): n_periodic adapters (a seeded choice among all ids) each have a period
    T (drawn from `periods`) and a phase and are requested once or twice in every window t with
    (t + phase) % T == 0; the rest of each window of `window` requests is i.i.d. Zipf(s) background over
    all adapters.  Returns a list of n_windows int32 arrays (requests of a window in random order)."""
    ids = rng.permutation(population)[:n_periodic]
    T = rng.choice(np.asarray(periods), size=n_periodic)
    phase = rng.integers(0, 1 << 16, size=n_periodic) % T
    twice = rng.random(n_periodic) < 0.25
    p = zipf_probs(population, s)
    out = []
    for t in range(n_windows):
        active = (t + phase) % T == 0
        req = np.concatenate([ids[active], ids[active & twice]])
        if len(req) > window:
            req = req[:window]
        back = rng.choice(population, size=window - len(req), p=p)
        win = np.concatenate([req, back]).astype(np.int32)
        rng.shuffle(win)
        out.append(win)
    return out
