"""Pins for the oracle's batch translation and LoRA delta (no GPU).

The delta is Eq. 1 of the paper (Sec. II-A): the adapter adds B (A x).  The checks compare the
paged, per-token oracle against things outside it: numpy's stable argsort, a dense fp64
x (A^T B) built from the un-paged matrices, a library GEMM for the one-adapter special case, and
invariances that hold for the definition (zero scale, evict + reload onto other pages, token
permutation, zero-padding the rank, power-of-two scales, page-size independence, output RMS of
the small workload).  Non-square slots and distinct d_in / d_out make a transposed operand or a
swapped offset fail the dense check.
"""
import numpy as np
import pytest
import torch

from workload import (CONFIGS, DT_BF16, DT_F16, DT_F32, Layout, RAW_DTYPE, config_layout, draw_tok2adapter,
                      from_elt, make_act, make_adapter, make_adapters, slot_views, to_elt)


def _dense_delta(lay, blobs, ranks, scales, slot, x_raw, t2a):
    """fp64: delta[t] = scale_i * x[t] @ (A_i^T B_i), from the un-paged blob views."""
    x = from_elt(x_raw, lay.dtype).astype(np.float64)
    out = np.zeros((len(t2a), lay.d_out[slot]))
    for t, i in enumerate(t2a):
        if i < 0:
            continue
        A, B = slot_views(lay, ranks[i], blobs[i])[slot]
        W = from_elt(A, lay.dtype).astype(np.float64).T @ from_elt(B, lay.dtype).astype(np.float64)
        out[t] = scales[i] * (x[t] @ W)
    return out


def _oracle_delta(pool, lay, slot, x_raw, t2a, acc64, y0=None):
    T = len(t2a)
    y = np.zeros((T, lay.d_out[slot]), dtype=RAW_DTYPE[lay.dtype]) if y0 is None else y0.copy()
    v = pool.shrink(slot, x_raw, t2a, acc64=acc64)
    pool.expand(slot, v, t2a, y, acc64=acc64)
    return v, y


def _setup(oracle_mod, lay, ranks, scales, P, n_pages, seed, order=None):
    pool = oracle_mod.OraclePool(P, n_pages, lay.d_in, lay.d_out, lay.dtype, len(ranks), max(ranks))
    blobs = make_adapters(seed, lay, ranks)
    for i in (order if order is not None else range(len(ranks))):
        pool.load(i, ranks[i], scales[i], blobs[i])
    return pool, blobs


@pytest.mark.parametrize("T,n_ad", [(0, 3), (1, 1), (17, 5), (1000, 37), (4096, 600)])
def test_translate_equals_numpy_stable_argsort(oracle_mod, T, n_ad):
    rng = np.random.default_rng(T + n_ad)
    lay = Layout((8,), (8,), DT_F16)
    pool = oracle_mod.OraclePool(4096, max(n_ad, 1), lay.d_in, lay.d_out, DT_F16, 700, 4)
    ids = rng.choice(700, size=n_ad, replace=False)
    for i in ids:
        pool.load(int(i), 1, 1.0, np.zeros(16, np.uint16))
    t2a = draw_tok2adapter(rng, T, ids, s=1.0, none_frac=0.2)
    perm, seg_adapter, seg_start = pool.translate(t2a)
    keep = np.nonzero(t2a >= 0)[0]
    ref_perm = keep[np.argsort(t2a[keep], kind="stable")]
    assert perm.tolist() == ref_perm.tolist()
    uniq, counts = np.unique(t2a[keep], return_counts=True)
    assert seg_adapter.tolist() == uniq.tolist()
    assert seg_start.tolist() == np.concatenate([[0], np.cumsum(counts)]).tolist()


def test_translate_rejects_non_resident(oracle_mod):
    lay = Layout((8,), (8,), DT_F16)
    pool = oracle_mod.OraclePool(4096, 4, lay.d_in, lay.d_out, DT_F16, 8, 4)
    pool.load(2, 1, 1.0, np.zeros(16, np.uint16))
    with pytest.raises(oracle_mod.OracleError) as ei:
        pool.translate(np.array([2, 3], np.int32))
    assert ei.value.code == -4
    with pytest.raises(oracle_mod.OracleError) as ei:
        pool.translate(np.array([2, 9], np.int32))
    assert ei.value.code == -1


@pytest.mark.parametrize("dtype", [DT_F16, DT_BF16, DT_F32])
@pytest.mark.parametrize("acc64", [False, True])
def test_delta_equals_dense_fp64(oracle_mod, dtype, acc64):
    """Brute force against Eq. 1 on tiny, non-square, multi-slot shapes with ragged ranks."""
    lay = Layout((24, 40, 16), (56, 8, 32), dtype)
    ranks, scales = [1, 3, 8, 5], [0.5, 2.0, -1.25, 3.0]
    pool, blobs = _setup(oracle_mod, lay, ranks, scales, 4096, 16, seed=5, order=[2, 0, 3, 1])
    rng = np.random.default_rng(9)
    t2a = np.array([3, 0, -1, 2, 2, 1, 0, 3, -1, 1, 2], dtype=np.int32)
    for slot in range(lay.n_slots):
        x = make_act(rng, len(t2a), lay.d_in[slot], dtype)
        v, y = _oracle_delta(pool, lay, slot, x, t2a, acc64)
        ref = _dense_delta(lay, blobs, ranks, scales, slot, x, t2a)
        got = from_elt(y, dtype).astype(np.float64)
        scale_ref = np.sqrt((ref ** 2).mean())
        tol = {DT_F32: 1e-5 if not acc64 else 2e-7, DT_F16: 1.2e-3, DT_BF16: 9e-3}[dtype]  # output rounding
        assert np.abs(got - ref).max() <= tol * max(scale_ref, 1.0) * 4
        assert (got[t2a < 0] == 0).all()
        # v itself: x A^T, before any output rounding
        for t, i in enumerate(t2a):
            if i < 0:
                assert (v[t] == 0).all()
                continue
            A = from_elt(slot_views(lay, ranks[i], blobs[i])[slot][0], dtype).astype(np.float64)
            vr = A @ from_elt(x[t], dtype).astype(np.float64)
            assert np.allclose(v[t, :ranks[i]], vr, rtol=0, atol=(1e-12 if acc64 else 2e-5) * max(1, np.abs(vr).max()))
            assert (v[t, ranks[i]:] == 0).all()


def test_single_adapter_one_page_is_a_plain_gemm(oracle_mod):
    """One adapter, page >= adapter: the path degenerates to two library GEMMs."""
    lay = Layout((256,), (192,), DT_F32)
    r, scale, T = 16, 0.75, 33
    pool, blobs = _setup(oracle_mod, lay, [r], [scale], 1 << 16, 1, seed=3)
    assert lay.adapter_bytes(r) <= 1 << 16
    rng = np.random.default_rng(4)
    x = make_act(rng, T, 256, DT_F32)
    t2a = np.zeros(T, np.int32)
    v, y = _oracle_delta(pool, lay, 0, x, t2a, acc64=False)
    A, B = slot_views(lay, r, blobs[0])[0]
    ref = scale * (torch.from_numpy(x) @ torch.from_numpy(A).T @ torch.from_numpy(B)).numpy()
    assert np.abs(y - ref).max() <= 1e-5 * np.sqrt((ref ** 2).mean()) * 4


def _standard(oracle_mod, dtype=DT_BF16, P=4096, scales=None, order=None, ranks=(4, 16, 9, 32), n_pages=64):
    lay = Layout((128, 64), (96, 160), dtype)
    ranks = list(ranks)
    scales = scales if scales is not None else [16.0 / r for r in ranks]
    pool, blobs = _setup(oracle_mod, lay, ranks, scales, P, n_pages, seed=21, order=order)
    rng = np.random.default_rng(22)
    t2a = draw_tok2adapter(rng, 40, np.arange(len(ranks)), s=1.0, none_frac=0.1)
    xs = [make_act(rng, 40, lay.d_in[s], dtype) for s in range(2)]
    y0 = [make_act(rng, 40, lay.d_out[s], dtype) for s in range(2)]
    return lay, ranks, scales, pool, blobs, t2a, xs, y0


def test_zero_scale_gives_zero_delta(oracle_mod):
    lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod, scales=[0.0, 0.0, 0.0, 0.0])
    for s in range(2):
        _, y = _oracle_delta(pool, lay, s, xs[s], t2a, False)
        assert (from_elt(y, lay.dtype) == 0).all()
        _, y = _oracle_delta(pool, lay, s, xs[s], t2a, False, y0=y0[s])
        assert (y == y0[s]).all()


def test_evict_and_reload_on_other_pages_is_bit_identical(oracle_mod):
    lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod)
    before = [_oracle_delta(pool, lay, s, xs[s], t2a, False, y0=y0[s]) for s in range(2)]
    pt_old = pool.page_table(1)
    pool.evict(0)
    pool.evict(1)
    pool.load(1, ranks[1], scales[1], blobs[1])  # lands on adapter 0's old pages first
    pool.load(0, ranks[0], scales[0], blobs[0])
    assert pool.page_table(1).tolist() != pt_old.tolist()
    after = [_oracle_delta(pool, lay, s, xs[s], t2a, False, y0=y0[s]) for s in range(2)]
    for (v0, ya), (v1, yb) in zip(before, after):
        assert (v0.view(np.uint32) == v1.view(np.uint32)).all() and (ya == yb).all()


def test_token_permutation_permutes_rows(oracle_mod):
    lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod)
    perm = np.random.default_rng(1).permutation(len(t2a))
    for s in range(2):
        v, y = _oracle_delta(pool, lay, s, xs[s], t2a, False, y0=y0[s])
        vp, yp = _oracle_delta(pool, lay, s, xs[s][perm], t2a[perm], False, y0=y0[s][perm])
        assert (vp.view(np.uint32) == v[perm].view(np.uint32)).all() and (yp == y[perm]).all()


def test_zero_padding_the_rank_is_bit_identical(oracle_mod):
    """An adapter of rank r and the same adapter zero-padded to rank r' give the same delta."""
    lay = Layout((128,), (96,), DT_BF16)
    r, rp = 5, 12
    rng = np.random.default_rng(2)
    blob = make_adapter(rng, lay, r)
    A, B = slot_views(lay, r, blob)[0]
    padded = np.zeros(lay.adapter_elems(rp), np.uint16)
    Ap, Bp = slot_views(lay, rp, padded)[0]
    Ap[:r], Bp[:r] = A, B
    pool = oracle_mod.OraclePool(4096, 8, lay.d_in, lay.d_out, DT_BF16, 2, rp)
    pool.load(0, r, 1.5, blob)
    pool.load(1, rp, 1.5, padded)
    x = make_act(rng, 7, 128, DT_BF16)
    y0 = make_act(rng, 7, 96, DT_BF16)
    _, ya = _oracle_delta(pool, lay, 0, x, np.zeros(7, np.int32), False, y0=y0)
    _, yb = _oracle_delta(pool, lay, 0, x, np.ones(7, np.int32), False, y0=y0)
    assert (ya == yb).all()


def test_power_of_two_scale_is_exact(oracle_mod):
    a = _standard(oracle_mod, dtype=DT_F32, scales=[1.0] * 4)
    b = _standard(oracle_mod, dtype=DT_F32, scales=[2.0] * 4)
    for s in range(2):
        _, y1 = _oracle_delta(a[3], a[0], s, a[6][s], a[5], False)
        _, y2 = _oracle_delta(b[3], b[0], s, b[6][s], b[5], False)
        assert (y2 == 2.0 * y1).all() and np.abs(y1).max() > 0


def test_page_size_independence(oracle_mod):
    ref = None
    for P, n_pages in [(4096, 64), (8192, 32), (65536, 8), (2 << 20, 4)]:
        lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod, P=P, n_pages=n_pages)
        out = [_oracle_delta(pool, lay, s, xs[s], t2a, False, y0=y0[s])[1] for s in range(2)]
        if ref is None:
            ref = out
        for a, b in zip(ref, out):
            assert (a == b).all()


def test_fp32_and_fp64_accumulation_agree(oracle_mod):
    lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod, dtype=DT_F32)
    for s in range(2):
        _, y32 = _oracle_delta(pool, lay, s, xs[s], t2a, False)
        _, y64 = _oracle_delta(pool, lay, s, xs[s], t2a, True)
        assert np.abs(y32 - y64).max() <= 1e-5 * np.sqrt((y64.astype(np.float64) ** 2).mean())


def test_small_workload_output_rms(oracle_mod):
    """1024->1024 fp16, A ~ N(0, 1/1024) (variance), B ~ N(0, 1/r), x ~ N(0,1), scale 2:
    v ~ N(0,1) and the delta has RMS ~ scale = 2."""
    cfg = CONFIGS["cfg0"]
    lay = config_layout(cfg)
    ranks, scales = cfg["ranks"], [cfg["scale"]] * 4
    pool, blobs = _setup(oracle_mod, lay, ranks, scales, cfg["page_bytes"], cfg["n_pages"], seed=cfg["seed"])
    rng = np.random.default_rng(cfg["seed"])
    t2a = draw_tok2adapter(rng, 256, np.arange(4), s=None)  # more tokens than the workload, same law
    x = make_act(rng, 256, 1024, DT_F16)
    v, y = _oracle_delta(pool, lay, 0, x, t2a, False)
    vr = np.concatenate([v[t, :ranks[i]] for t, i in enumerate(t2a)])
    assert abs(np.sqrt((vr.astype(np.float64) ** 2).mean()) - 1.0) < 0.05
    rms = np.sqrt((from_elt(y, DT_F16).astype(np.float64) ** 2).mean())
    assert abs(rms - 2.0) < 0.1


def test_token_subset_matches_full_run(oracle_mod):
    lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod)
    sel = np.array([3, 17, 39, 0], np.int32)
    v = pool.shrink(0, xs[0], t2a, acc64=True)
    vs = pool.shrink(0, xs[0], t2a, acc64=True, tok_sel=sel)
    assert (v[sel] == vs[sel]).all()
    y = pool.expand(0, v, t2a, y0[0].copy(), acc64=True)
    ys = pool.expand(0, vs, t2a, y0[0].copy(), acc64=True, tok_sel=sel)
    assert (y[sel] == ys[sel]).all()
    rest = np.setdiff1d(np.arange(len(t2a)), sel)
    assert (ys[rest] == y0[0][rest]).all()


def test_threads_do_not_change_results(oracle_mod):
    lay, ranks, scales, pool, blobs, t2a, xs, y0 = _standard(oracle_mod)
    v1 = pool.shrink(1, xs[1], t2a)
    v4 = pool.shrink(1, xs[1], t2a, threads=4)
    assert (v1.view(np.uint32) == v4.view(np.uint32)).all()
    y1 = pool.expand(1, v1, t2a, y0[1].copy())
    y4 = pool.expand(1, v4, t2a, y0[1].copy(), threads=4)
    assert (y1 == y4).all()
