"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

from workload import (CONFIGS, DT_BF16, DT_F16, DT_F32, Layout, config_layout, draw_tok2adapter, from_elt)
from helpers import Case

pytestmark = pytest.mark.gpu


def test_cfg0_small_workload(oracle_mod):
    """1024->1024 fp16, 16 tokens, ranks (8,16,8,16), scale 2, 16 KiB pages, 64 pages."""
    cfg = CONFIGS["cfg0"]
    lay = config_layout(cfg)
    case = Case(oracle_mod, lay, cfg["ranks"], [cfg["scale"]] * 4, cfg["page_bytes"], cfg["n_pages"], cfg["seed"])
    rng = np.random.default_rng(cfg["seed"])
    t2a = draw_tok2adapter(rng, cfg["tokens"], np.arange(4), s=None)
    print("cfg0 t2a", t2a.tolist(), flush=True)
    for mfma, major, remap in ((0, -1, 1), (1, 0, 1), (4, 1, 1), (2, 0, 0), (1, 1, 0)):
        case.set_mfma(mfma, 0 if mfma == 4 else mfma)
        if major >= 0:  # -1: the library's own geometry (shrink: slots fastest if a multiple of 8, expand: chunks fastest)
            case.gpool.set_option("slot_major", major)
        case.gpool.set_option("xcd_remap", remap)
        out = case.run(t2a, seed=1)
        print("mfma_min", mfma, "err_v %.3g err_y %.3g" % (out[0]["err_v"], out[0]["err_y"]), flush=True)
        out = case.run(t2a, seed=2, y0_zero=True)
    st = case.gpool.stats()
    assert st["used_pages"] == 12
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F16, DT_F32])
@pytest.mark.parametrize("mfma,major", [(0, -1), (1, 0), (3, 1)])
def test_ragged_multi_slot(oracle_mod, dtype, mfma, major):
    """Several tiles and ragged tails everywhere: d not a multiple of the wave width, ranks 1..40
    (not multiples of 8), rows straddling 4 KiB pages, tokens without adapter, scattered pages."""
    lay = Layout((1000, 520, 72), (264, 1304, 8), dtype)
    ranks = [1, 3, 8, 17, 40, 5, 33, 16]
    scales = [16.0 / r for r in ranks]
    case = Case(oracle_mod, lay, ranks, scales, 4096, 1024, seed=77, load_order=[4, 0, 6, 2, 1, 7, 3, 5],
                mfma_min_tokens=mfma)
    if major >= 0:
        case.gpool.set_option("slot_major", major)
    # scatter: evict two adapters and reload them so that their pages interleave
    case.evict(0)
    case.evict(6)
    case.load(6)
    case.load(0)
    rng = np.random.default_rng(5)
    for T in (1, 7, 90, 300):
        t2a = draw_tok2adapter(rng, T, np.arange(len(ranks)), s=1.0, none_frac=0.15)
        print("ragged dtype", dtype, "mfma", mfma, "T", T, flush=True)
        out = case.run(t2a, seed=T)
        print("   err_v", ["%.2g" % o["err_v"] for o in out], "err_y", ["%.2g" % o["err_y"] for o in out], flush=True)
    case.close()


def test_empty_and_no_adapter_batches(oracle_mod):
    lay = Layout((64,), (64,), DT_BF16)
    case = Case(oracle_mod, lay, [4], [1.0], 4096, 4, seed=1)
    case.run(np.zeros(0, np.int32))
    case.run(np.full(9, -1, np.int32))
    case.close()


def test_evict_reload_bit_identical_on_gpu(oracle_mod):
    lay = Layout((512, 256), (256, 768), DT_BF16)
    ranks = [8, 16, 24, 64]
    case = Case(oracle_mod, lay, ranks, [2.0, 1.0, 0.5, 0.25], 4096, 256, seed=9, mfma_min_tokens=6)
    rng = np.random.default_rng(3)
    t2a = draw_tok2adapter(rng, 64, np.arange(4), s=1.0)
    a = case.run(t2a, seed=4)
    case.evict(0)
    case.evict(2)
    case.load(2)
    case.load(0)
    b = case.run(t2a, seed=4)
    for ra, rb in zip(a, b):
        assert (ra["v_got"].view(np.uint32) == rb["v_got"].view(np.uint32)).all()
        assert (ra["y_got"] == rb["y_got"]).all()
    case.close()


def test_error_paths_on_gpu(oracle_mod):
    import torch
    import paper_2512_20210_amd as P
    lay = Layout((64,), (64,), DT_BF16)
    case = Case(oracle_mod, lay, [4, 8], [1.0, 1.0], 4096, 2, seed=1, max_adapters=4, load_order=[0])
    g = case.gpool
    # not enough pages: nothing allocated
    rc, _ = P.plora_load_adapter(g.h, 1, 8, 1.0, case.pinned[1].data_ptr(), None)
    assert rc == P.PLORA_OK  # 8*128*2 = 2 KiB -> 1 page
    rc, _ = P.plora_load_adapter(g.h, 2, 8, 1.0, case.pinned[1].data_ptr(), None)
    assert rc == P.PLORA_ERR_NOMEM and g.stats()["free_pages"] == 0
    rc, _ = P.plora_load_adapter(g.h, 1, 8, 1.0, case.pinned[1].data_ptr(), None)
    assert rc == P.PLORA_ERR_EXISTS
    unpinned = torch.zeros(4096, dtype=torch.int16)
    assert P.plora_evict(g.h, 1) == P.PLORA_OK or P.plora_evict(g.h, 1) == P.PLORA_ERR_BUSY
    torch.cuda.synchronize()
    if P.plora_adapter_ready(g.h, 1) != P.PLORA_ERR_NOTFOUND:
        assert P.plora_evict(g.h, 1) == P.PLORA_OK
    rc, _ = P.plora_load_adapter(g.h, 1, 8, 1.0, unpinned.data_ptr(), None)
    assert rc == P.PLORA_ERR_INVAL and g.stats()["free_pages"] == 1
    rc, b = P.plora_batch_begin(g.h, np.array([0, 3], np.int32), None)
    assert rc == P.PLORA_ERR_NOTFOUND
    rc, b = P.plora_batch_begin(g.h, np.array([0, 7], np.int32), None)
    assert rc == P.PLORA_ERR_INVAL
    rc, b = P.plora_batch_begin(g.h, np.array([0, 0], np.int32), None)
    assert rc == P.PLORA_OK
    assert P.plora_evict(g.h, 0) == P.PLORA_ERR_BUSY       # pinned by the open batch
    assert P.plora_pool_destroy(g.h) == P.PLORA_ERR_BUSY
    x = torch.zeros(2, 64, dtype=torch.int16, device="cuda")
    v = torch.zeros(2, 8, dtype=torch.float32, device="cuda")
    assert P.plora_shrink(g.h, b, 0, 2, [x.data_ptr()] * 2, [v.data_ptr()] * 2, None) == P.PLORA_ERR_INVAL  # slot range
    assert P.plora_shrink(g.h, b, 0, 1, [x.data_ptr() + 2], [v.data_ptr()], None) == P.PLORA_ERR_INVAL      # alignment
    assert P.plora_batch_end(g.h, b) == P.PLORA_OK
    torch.cuda.synchronize()
    assert P.plora_evict(g.h, 0) == P.PLORA_OK
    assert P.plora_evict(g.h, 0) == P.PLORA_ERR_NOTFOUND
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F16])
def test_large_groups_panels_and_odd_strides(oracle_mod, dtype):
    """Prefill-like groups (hundreds of tokens per adapter) through the token-split matrix-core
    expand and the split-K matrix-core shrink, with a row stride of v that is not a multiple of 4,
    ragged widths and ranks, 2 MiB pages (the paper's default page size)."""
    lay = Layout((1096, 328), (712, 1544), dtype)
    ranks = [37, 8, 64, 19, 3]
    scales = [16.0 / r for r in ranks]
    case = Case(oracle_mod, lay, ranks, scales, 2 << 20, 8, seed=31, max_rank=67, mfma_min_tokens=5)
    rng = np.random.default_rng(8)
    # group sizes 1, 7, 33, 70, 260: vector-ALU, column-split, and token-split items
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in zip(range(5), (260, 70, 33, 7, 1))])
    rng.shuffle(t2a)
    for major in (-1, 1):
        if major >= 0:  # first pass: the library's own geometry
            case.gpool.set_option("slot_major", major)
        out = case.run(t2a, seed=3)
        print("panels dtype", dtype, "slot_major", major, "err_v", ["%.2g" % o["err_v"] for o in out],
              "err_y", ["%.2g" % o["err_y"] for o in out], flush=True)
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F16])
def test_panel_kernel_forms_agree_bit_for_bit(oracle_mod, dtype):
    """The panel kernel with one workgroup per 512 columns and with one per 256 (option
    panel_half_max_workgroups) forms every element of y by the same sequence of operations: same bits.
    Widths that end inside the first half, inside the second, and on their boundaries."""
    lay = Layout((264, 520, 128, 256), (200, 776, 256, 512), dtype)
    ranks = [64, 24, 130, 7]
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], 64 << 10, 48, seed=77, max_rank=130, mfma_min_tokens=5)
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in zip(range(4), (200, 150, 90, 64))])
    np.random.default_rng(9).shuffle(t2a)
    got = []
    for half in (0, 1 << 40):
        case.kernel_modes = ((0, 1, 0, "pair", half),)
        out = case.run(t2a, seed=4)
        got.append([o["y_got"].copy() for o in out])
    for s, (y_full, y_half) in enumerate(zip(*got)):
        assert (y_full.view(np.uint16) == y_half.view(np.uint16)).all(), "slot %d: the two forms differ" % s
    case.close()


def test_many_small_adapters_64k_pages(oracle_mod):
    """200 adapters of ranks 1..16 on 64 KiB pages, most tokens alone with their adapter."""
    lay = Layout((512,), (1024,), DT_BF16)
    rng = np.random.default_rng(12)
    ranks = rng.integers(1, 17, size=200).tolist()
    case = Case(oracle_mod, lay, ranks, [1.0] * 200, 65536, 200, seed=13)
    t2a = draw_tok2adapter(rng, 333, np.arange(200), s=0.7, none_frac=0.05)
    out = case.run(t2a, seed=1)
    print("small adapters err_v %.2g err_y %.2g" % (out[0]["err_v"], out[0]["err_y"]), flush=True)
    case.close()


def test_slots_of_two_widths_in_one_call(oracle_mod):
    """16 slots, 8 of them 512 columns wide and 8 of them 1536 (as with grouped-query k, v next to
    q, o): the expand call runs one launch per width; plus a 12-slot call (classes of 6: one launch)."""
    d_out = (512, 1536, 1536, 512) * 4
    lay = Layout((256,) * 16, d_out, DT_BF16)
    ranks = [8, 24, 64, 5]
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], 16384, 512, seed=53)
    rng = np.random.default_rng(8)
    t2a = draw_tok2adapter(rng, 70, np.arange(len(ranks)), s=1.0, none_frac=0.1)
    for mfma in (0, 4):
        case.set_mfma(mfma)
        case.run(t2a, seed=3)
        case.run(t2a, slots=range(2, 14), seed=4)
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F16])
def test_matrix_core_shrink_with_one_and_two_runs_in_flight(oracle_mod, dtype):
    """Contractions of 1 .. 67 runs of 64 values (so the four wavefronts of an item get 0, 1, 2, 3,
    even and odd numbers of runs), ragged last runs, full and ragged token tiles: both depths against
    the oracle, and against each other bit for bit (the order of the sums is the same)."""
    d_ins = (64, 72, 128, 192, 200, 448, 456, 640, 1000, 4096, 4288)
    lay = Layout(d_ins, (64,) * len(d_ins), dtype)
    ranks = [8, 24, 32, 64, 40]
    case = Case(oracle_mod, lay, ranks, [1.0] * len(ranks), 4096, 4096, seed=77)
    case.set_mfma(1)
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in ((0, 1), (1, 32), (2, 33), (3, 70), (4, 5))])
    np.random.default_rng(78).shuffle(t2a)
    got = {}
    for depth in (1, 2):
        case.kernel_modes = ((0, 8, depth, "pair"),)
        out = case.run(t2a, seed=3)
        got[depth] = [o["v_got"].copy() for o in out]
    for a, b in zip(got[1], got[2]):
        assert (a.view(np.uint32) == b.view(np.uint32)).all()
    case.close()


def test_slots_that_share_one_x_buffer(oracle_mod):
    """q, k and v of a layer read the same x: slots of a call may be given one buffer."""
    lay = Layout((256, 256, 256, 256, 200, 200, 128), (64, 128, 64, 64, 64, 72, 64), DT_BF16)
    ranks = [8, 24, 32, 64, 40]
    case = Case(oracle_mod, lay, ranks, [1.0] * len(ranks), 4096, 2048, seed=81)
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in ((0, 1), (1, 32), (2, 33), (3, 70), (4, 5))] + [np.full(3, -1, np.int32)])
    np.random.default_rng(82).shuffle(t2a)
    for mfma in (1, 0):
        case.set_mfma(mfma)
        case.run(t2a, seed=4, share_x=((0, 1, 2, 3), (4, 5)))
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F32])
def test_maximum_rank(oracle_mod, dtype):
    """Ranks up to the library's limit of 512 (the expand stages one page pair per row of B), with
    groups small and large enough for every kind of item."""
    lay = Layout((136, 64), (72, 520), dtype)
    ranks = [512, 300, 509, 8]
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], 8192, 1024, seed=61, max_rank=512)
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in zip(range(4), (70, 3, 18, 1))])
    np.random.default_rng(2).shuffle(t2a)
    for mfma in (0, 2):
        case.set_mfma(mfma)
        out = case.run(t2a, seed=7)
        print("max rank dtype", dtype, "mfma", mfma, "err_v", ["%.2g" % o["err_v"] for o in out],
              "err_y", ["%.2g" % o["err_y"] for o in out], flush=True)
    case.close()


@pytest.mark.parametrize("per_marker", [1, 4, 64])
def test_pages_freed_behind_queued_batches_are_rewritten_only_after_their_kernels(oracle_mod, per_marker):
    """Three batches that read adapter 0 are queued, the adapter is evicted and another one is loaded
    onto the same pages without any synchronisation in between: the copy has to wait for the batches'
    kernels whether or not their completion event had been put on the stream yet."""
    import torch
    from workload import from_elt, make_act
    from helpers import TOL_Y, raw_to_torch, rel_err, torch_to_raw
    lay = Layout((4096,) * 8, (4096,) * 8, DT_BF16)
    ranks = [64, 64]
    case = Case(oracle_mod, lay, ranks, [0.5, 2.0], 65536, 2 * 128 + 8, seed=21, load_order=[0])
    g, o = case.gpool, case.opool
    g.set_option("batches_per_marker", per_marker)
    T, rng = 512, np.random.default_rng(8)
    slots = list(range(lay.n_slots))
    runs = []
    for k in range(4):  # three batches over adapter 0, then one over adapter 1
        xs = [make_act(rng, T, lay.d_in[s], lay.dtype) for s in slots]
        y0 = [make_act(rng, T, lay.d_out[s], lay.dtype) for s in slots]
        runs.append(dict(xs=xs, y0=y0, xd=[raw_to_torch(a, "cuda") for a in xs], yd=[raw_to_torch(a, "cuda") for a in y0],
                         vd=[torch.empty((T, 64), device="cuda") for _ in slots]))
    torch.cuda.synchronize()
    t2a0, t2a1 = np.zeros(T, np.int32), np.ones(T, np.int32)
    sel = np.arange(0, T, 37, dtype=np.int32)

    def reference(r, t2a):
        r["ref"] = []
        for s in slots:
            v_ref = o.shrink(s, r["xs"][s], t2a, acc64=True, tok_sel=sel)
            r["ref"].append(o.expand(s, v_ref, t2a, r["y0"][s].copy(), acc64=True, tok_sel=sel))

    def gpu(r, t2a):
        b = g.batch_begin(t2a, case.stream)
        g.shrink(b, 0, r["xd"], r["vd"], case.stream)
        g.expand(b, 0, r["vd"], r["yd"], case.stream)
        g.batch_end(b)

    for r in runs[:3]:
        reference(r, t2a0)
    print("per_marker", per_marker, "queueing three batches, evict, load, one batch", flush=True)
    for r in runs[:3]:
        gpu(r, t2a0)
    pt0 = o.page_table(0).tolist()
    case.evict(0)
    pt1 = case.load(1)
    assert pt1.tolist() == pt0, "the new adapter did not land on the freed pages"
    gpu(runs[3], t2a1)
    torch.cuda.synchronize()
    reference(runs[3], t2a1)
    for k, r in enumerate(runs):
        for s in slots:
            got = torch_to_raw(r["yd"][s], lay.dtype)
            err = rel_err(from_elt(got[sel], lay.dtype), from_elt(r["ref"][s][sel], lay.dtype))
            assert err <= TOL_Y[lay.dtype], "batch %d slot %d: y error %.3g" % (k, s, err)
    assert g.stats()["used_pages"] == 128
    case.close()


@pytest.mark.parametrize("page_bytes,dims,filler_rank,big_ranks", [
    (16384, ((4096,), (4096,)), 1, (64, 512, 200)),      # 64, 512 (three scatter launches) and 200 single-page runs
    (65536, ((1024, 1024), (1024, 1024)), 8, (24, 51)),   # last page partly filled: one and a half 16 KiB pieces
    (4096, ((64,), (64,)), 16, (100, 7)),                 # pages smaller than the piece one workgroup moves
])
def test_staged_loads_put_the_same_bytes_in_the_same_pages(oracle_mod, page_bytes, dims, filler_rank, big_ranks):
    """Staged load (one copy into a staging buffer + scatter kernel) on a pool whose free pages are
    single-page holes: page tables as the oracle's, slab bytes through the tables identical to the
    blobs, and a batch over the staged adapters matches the oracle."""
    import torch
    lay = Layout(dims[0], dims[1], DT_BF16)
    C = sum(dims[0]) + sum(dims[1])
    pages_of = lambda r: -(-(r * 2 * C) // page_bytes)
    assert pages_of(filler_rank) == 1
    need = sum(pages_of(r) for r in big_ranks)
    n_fill = 2 * need + 2
    ranks = [filler_rank] * n_fill + list(big_ranks)
    n_pages = n_fill + 8
    slab = torch.zeros(n_pages * page_bytes, dtype=torch.uint8, device="cuda")
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], page_bytes, n_pages, seed=31,
                load_order=list(range(n_fill)), max_rank=max(ranks), slab=slab)
    g = case.gpool
    g.set_option("staging_bytes", max(big_ranks) * 2 * C)
    for i in range(0, n_fill, 2):
        case.evict(i)
    for k, r in enumerate(big_ranks):
        aid = n_fill + k
        print("staged load of rank", r, "=", pages_of(r), "pages of", page_bytes, flush=True)
        pt = case.load(aid)  # asserts that the table equals the oracle's
        assert len(pt) == pages_of(r)
    torch.cuda.synchronize()
    # the last adapter may have found the contiguous tail of the pool: count what went staged
    st = g.stats()
    assert st["staged_loads"] >= len(big_ranks) - 1, st
    pages = slab.view(n_pages, page_bytes).cpu().numpy()
    for k, r in enumerate(big_ranks):
        aid = n_fill + k
        S = r * 2 * C
        pt = case.opool.page_table(aid)
        got = pages[pt].reshape(-1)[:S]
        assert (got == case.blobs[aid].view(np.uint8).reshape(-1)).all(), "slab bytes of adapter %d differ from its blob" % aid
    # untouched neighbours: the fillers that stayed keep their bytes
    for i in range(1, n_fill, 2):
        pt = case.opool.page_table(i)
        S = filler_rank * 2 * C
        assert (pages[pt].reshape(-1)[:S] == case.blobs[i].view(np.uint8).reshape(-1)).all()
    rng = np.random.default_rng(4)
    ids = np.array([n_fill + k for k in range(len(big_ranks))] + [1, 3], dtype=np.int32)
    t2a = ids[rng.integers(0, len(ids), size=24)].astype(np.int32)
    case.run(t2a, seed=9)
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F16, DT_F32])
def test_zero_and_negative_scale_and_signed_zero_y(oracle_mod, dtype):
    """Scale 0 (the delta vanishes: y keeps its value, and only the sign of a zero may change), scale
    < 0, y0 = +0 and y0 = -0 everywhere; vector-ALU and matrix-core items (Eq. 1 with the per-adapter
    scale applied once in fp32)."""
    lay = Layout((520, 256), (264, 1024), dtype)
    ranks = [8, 16, 40, 64, 5]
    scales = [0.0, -2.0, -0.125, 0.0, 1.5]
    case = Case(oracle_mod, lay, ranks, scales, 8192, 256, seed=91)
    rng = np.random.default_rng(92)
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in zip(range(5), (21, 40, 3, 1, 18))] + [np.full(2, -1, np.int32)])
    rng.shuffle(t2a)
    minus_zero = np.float32(-0.0) if dtype == DT_F32 else np.uint16(0x8000)
    for mfma in (0, 2):
        case.set_mfma(mfma)
        for kw in (dict(), dict(y0_zero=True), dict(y0_fill=minus_zero)):
            out = case.run(t2a, seed=5, **kw)
            for o in out:
                zero_scale = np.isin(t2a, [0, 3])
                got, y0 = from_elt(o["y_got"], dtype), from_elt(o["y0"], dtype)
                # zero scale: y keeps its value, bit for bit, except that a -0 may come back as +0
                # (-0 + (+0) = +0; which zero the product 0 * acc is depends on the sign of acc)
                assert (got[zero_scale] == y0[zero_scale]).all()
                keeps_bits = (o["y_got"][zero_scale] == o["y0"][zero_scale]) | (y0[zero_scale] == 0)
                assert keeps_bits.all()
        print("scales dtype", dtype, "mfma", mfma, "ok", flush=True)
    case.close()


@pytest.mark.parametrize("dtype", [DT_BF16, DT_F16])
@pytest.mark.parametrize("x_std", [1.0 / 64, 64.0, 1e-4, 3e3])
def test_activations_far_from_unit_scale(oracle_mod, dtype, x_std):
    """v = x A^T scales with x: rows of v of magnitude 1e-4 .. 3e3 through the vector-ALU items and
    through the matrix-core expand, which feeds v to the matrix cores as 16-bit halves (fp16: after a
    per-row power-of-two scaling)."""
    lay = Layout((1024,), (520,), dtype)
    ranks = [8, 32, 64, 24]
    # a large scale on one adapter pushes |v| further out; y0 = 0 so that y itself stays finite in fp16
    case = Case(oracle_mod, lay, ranks, [1.0, 0.25, 1.0 / 64, 2.0], 16384, 64, seed=95)
    rng = np.random.default_rng(96)
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in zip(range(4), (17, 70, 5, 2))])
    rng.shuffle(t2a)
    if dtype == DT_F16 and x_std > 60:
        x_std = min(x_std, 600.0)  # x itself must stay below 65504 after 4-sigma draws
    for mfma in (0, 1):
        case.set_mfma(mfma)
        out = case.run(t2a, seed=6, x_std=x_std, y0_zero=True)
        vmax = float(np.abs(out[0]["v_ref"]).max())
        print("x_std %g dtype %d mfma %d: max|v| %.3g err_v %.2g err_y %.2g" % (x_std, dtype, mfma, vmax, out[0]["err_v"], out[0]["err_y"]), flush=True)
        assert np.isfinite(from_elt(out[0]["y_got"], dtype)).all() == np.isfinite(from_elt(out[0]["y_ref"], dtype)).all()
    case.close()


def test_fp16_rows_of_v_beyond_fp16_range(oracle_mod):
    """fp16 elements; rows of v from 2^-17 to 2^18 in one batch (fp16 itself holds 2^-14 .. 65504 with
    full precision): adapter 0 has A sixteen times the usual size and tokens of magnitude 2^-8 .. 2^14,
    adapter 1 has A a sixteenth of it and tokens of magnitude 2^-13 .. 2^-11; the adapters' scales
    bring the deltas back into fp16's range.  The matrix-core expand must neither overflow the large
    rows nor lose the small ones (each row has its own power-of-two scale), checked row by row."""
    from workload import make_adapters, slot_views, to_elt
    from helpers import rel_err
    lay = Layout((4096,), (512,), DT_F16)
    ranks = [32, 16]
    blobs = make_adapters(97, lay, ranks)
    for blob, r, f in zip(blobs, ranks, (16.0, 1.0 / 16)):
        A, _ = slot_views(lay, r, blob)[0]
        A[:] = to_elt(from_elt(A, DT_F16) * np.float32(f), DT_F16)
    case = Case(oracle_mod, lay, ranks, [2.0 ** -8, 2.0 ** 12], 16384, 64, seed=97, blobs=blobs)
    case.set_mfma(1)
    T0, T1 = 40, 9
    t2a = np.concatenate([np.zeros(T0, np.int32), np.ones(T1, np.int32)])
    rng = np.random.default_rng(98)
    mags = np.concatenate([np.float32(2.0) ** rng.integers(-8, 15, size=T0).astype(np.float32),
                           np.float32(2.0) ** rng.integers(-13, -10, size=T1).astype(np.float32)])
    mags[0], mags[1] = 2.0 ** 14, 2.0 ** -8
    order = rng.permutation(T0 + T1)
    t2a, mags = t2a[order], mags[order]
    x = np.clip(rng.standard_normal((T0 + T1, 4096), dtype=np.float32), -3.5, 3.5) * mags[:, None]
    xs = [to_elt(x, DT_F16)]
    y0 = [np.zeros((T0 + T1, 512), np.uint16)]
    for coop, panel, depth, api in ((0, 8, 0, "pair"), (0, 1, 2, "delta")):
        case.gpool.set_option("coop_max_workgroups_shrink", coop)
        case.gpool.set_option("coop_max_workgroups_expand", coop)
        case.gpool.set_option("panel_min_blocks", panel)
        case.gpool.set_option("mfma_shrink_depth", depth)
        out = case._run_gpu(t2a, [0], xs, y0, False, api)[0]
        vmax = np.abs(out["v_ref"]).max(axis=1)
        print("fp16 wide rows (panel_min_blocks %d): max|v| per token from %.3g to %.3g" % (panel, vmax.min(), vmax.max()), flush=True)
        assert vmax.max() > 4 * 65504 and vmax.min() < 2.0 ** -14
        got, ref = from_elt(out["y_got"], DT_F16), from_elt(out["y_ref"], DT_F16)
        assert np.isfinite(ref).all() and np.isfinite(got).all()
        worst = max(rel_err(got[t], ref[t]) for t in range(T0 + T1))
        print("   worst row error %.3g" % worst, flush=True)
        for t in range(T0 + T1):
            assert rel_err(got[t], ref[t]) <= 1e-2, "token %d (max|v| %.3g): %.3g" % (t, vmax[t], rel_err(got[t], ref[t]))
    case.close()
