"""Shared test plumbing: build both sides from the same seeded inputs, run them, compare.

The comparison measure for float outputs is  max_i |got_i - ref_i| / max(|ref_i|, rms(ref)):
element-wise relative error with an rms floor so that outputs near zero do not blow it up.
Tolerances: 1e-2 for fp16 / bf16 storage with fp32 accumulation, 1e-5 for fp32; v (never rounded
to the element type) is held to 2e-5 against the fp64-accumulating oracle.
"""
import numpy as np

from workload import DT_F32, RAW_DTYPE, from_elt, make_act, make_adapters

TOL_Y = {0: 1e-2, 1: 1e-2, 2: 1e-5}
TOL_V = 2e-5


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt((ref ** 2).mean())
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float((np.abs(got - ref) / den).max())


def raw_to_torch(raw, device=None, pin=False):
    """Raw element array -> torch tensor of the same bytes (int16 / float32): plain memory."""
    import torch
    a = np.ascontiguousarray(raw)
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
    if pin:
        return t.pin_memory()
    return t.to(device) if device is not None else t


def torch_to_raw(t, dtype):
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if dtype != DT_F32 else a


class Case:
    """Oracle pool + GPU pool holding the same adapters (loaded in the same order)."""

    def __init__(self, oracle_mod, layout, ranks, scales, page_bytes, n_pages, seed, max_adapters=None,
                 max_rank=None, load_order=None, mfma_min_tokens=None, blobs=None, slab=None):
        import torch
        import paper_2512_20210_amd as P
        self.P, self.torch, self.lay = P, torch, layout
        self.ranks, self.scales = list(ranks), list(scales)
        self.max_rank = max_rank or max(ranks)
        na = max_adapters or len(ranks)
        self.blobs = blobs if blobs is not None else make_adapters(seed, layout, ranks)
        self.pinned = [raw_to_torch(b, pin=True) for b in self.blobs]
        self.opool = oracle_mod.OraclePool(page_bytes, n_pages, layout.d_in, layout.d_out, layout.dtype, na, self.max_rank)
        self.gpool = P.PagedLoraPool(page_bytes, n_pages, layout.d_in, layout.d_out, layout.dtype, na, self.max_rank, slab=slab)
        if mfma_min_tokens is not None:
            self.set_mfma(mfma_min_tokens)
        self.stream = torch.cuda.current_stream().cuda_stream
        self.copy_stream = torch.cuda.Stream()
        for i in (load_order if load_order is not None else range(len(ranks))):
            self.load(i)

    def set_mfma(self, n, n_expand=None):
        """Matrix-core items in shrink and in expand exactly for the adapter groups of at least n
        (n_expand) tokens, whatever their rank; 0 = never."""
        self.gpool.set_option("mfma_min_tokens", n)
        self.gpool.set_option("mfma_min_tokens_expand", n if n_expand is None else n_expand)
        self.gpool.set_option("mfma_min_work", 1 << 30)
        self.gpool.set_option("mfma_min_work_expand", 1 << 30)

    def load(self, i):
        pt_o = self.opool.load(i, self.ranks[i], self.scales[i], self.blobs[i])
        pt_g = self.gpool.load(i, self.ranks[i], self.scales[i], self.pinned[i], self.copy_stream.cuda_stream)
        assert pt_g.tolist() == pt_o.tolist(), "page tables differ for adapter %d" % i
        return pt_g

    def evict(self, i):
        self.opool.evict(i)
        self.gpool.evict(i)

    def run(self, t2a, slots=None, seed=0, y0_zero=False, check=True, x_std=1.0, share_x=(), y0_fill=None):
        """One batch over `slots` on both sides; returns per-slot dicts with raw outputs.  share_x:
        groups of positions in `slots` (same d_in) that read one x buffer, as q, k, v of a layer do.
        y0_fill: a raw element value that every entry of y0 takes (e.g. the bit pattern of -0)."""
        torch, lay = self.torch, self.lay
        t2a = np.ascontiguousarray(t2a, dtype=np.int32)
        T = len(t2a)
        slots = list(range(lay.n_slots)) if slots is None else list(slots)
        rng = np.random.default_rng(seed)
        xs = [make_act(rng, T, lay.d_in[s], lay.dtype, x_std) for s in slots]
        for group in share_x:
            for j in group[1:]:
                assert lay.d_in[slots[j]] == lay.d_in[slots[group[0]]]
                xs[j] = xs[group[0]]
        y0 = [np.zeros((T, lay.d_out[s]), RAW_DTYPE[lay.dtype]) if y0_zero else make_act(rng, T, lay.d_out[s], lay.dtype)
              for s in slots]
        if y0_fill is not None:
            y0 = [np.full_like(y, y0_fill) for y in y0]
        # GPU side: with the cooperative kernels of small calls, as two calls and through the one-call form
        # plora_delta (one launch over a task queue); with the panel kernel for every large group (as in a
        # prefill batch) and two runs in flight in every matrix-core shrink item, through plora_delta
        # (block lists in the one launch when the batch has no panel blocks); and with the library's own
        # choices last (its outputs are returned).  The panel kernel runs in both of its forms: one workgroup
        # per 512 columns, and one per 256.  Each entry: (cooperative limit, panel_min_blocks,
        # mfma_shrink_depth, entry points[, panel_half_max_workgroups; default: the library's 8192]).
        for mode in getattr(self, "kernel_modes", ((1 << 30, 8, 1, "pair"), (1 << 30, 8, 1, "delta"), (0, 1, 2, "delta", 0),
                                                   (0, 1, 1, "pair", 1 << 40), (0, 8, 0, "pair"))):
            coop, panel, depth, api = mode[:4]
            self.gpool.set_option("coop_max_workgroups_shrink", coop)
            self.gpool.set_option("coop_max_workgroups_expand", coop)
            self.gpool.set_option("panel_min_blocks", panel)
            self.gpool.set_option("panel_half_max_workgroups", mode[4] if len(mode) > 4 else 8192)
            self.gpool.set_option("mfma_shrink_depth", depth)
            self.gpool.set_option("fused_max_tasks", 1 << 20 if api == "delta" else 0)  # plora_delta as one launch where it applies
            out = self._run_gpu(t2a, slots, xs, y0, check, api)
        return out

    def _run_gpu(self, t2a, slots, xs, y0, check, api="pair"):
        torch, lay = self.torch, self.lay
        T = len(t2a)
        batch = self.gpool.batch_begin(t2a, self.stream)
        perm, seg_adapter, seg_start = self.gpool.batch_info(batch)
        o_perm, o_sa, o_ss = self.opool.translate(t2a)
        assert perm.tolist() == o_perm.tolist() and seg_adapter.tolist() == o_sa.tolist() and seg_start.tolist() == o_ss.tolist()
        on_device = {}
        xd = []
        for x in xs:  # one device buffer per distinct x
            if id(x) not in on_device:
                on_device[id(x)] = raw_to_torch(x, "cuda")
            xd.append(on_device[id(x)])
        yd = [raw_to_torch(y, "cuda") for y in y0]
        vd = [torch.full((max(T, 1), self.max_rank), float("nan"), device="cuda", dtype=torch.float32) for _ in slots]
        # contiguous slot runs go through one call each
        i = 0
        while i < len(slots):
            j = i
            while j + 1 < len(slots) and slots[j + 1] == slots[j] + 1:
                j += 1
            if api == "delta":
                self.gpool.delta(batch, slots[i], xd[i:j + 1], vd[i:j + 1], yd[i:j + 1], self.stream)
            else:
                self.gpool.shrink(batch, slots[i], xd[i:j + 1], vd[i:j + 1], self.stream)
                self.gpool.expand(batch, slots[i], vd[i:j + 1], yd[i:j + 1], self.stream)
            i = j + 1
        self.gpool.batch_end(batch)
        torch.cuda.synchronize()
        out = []
        for q, s in enumerate(slots):
            v_ref = self.opool.shrink(s, xs[q], t2a, acc64=True)
            y_ref = self.opool.expand(s, v_ref, t2a, y0[q].copy(), acc64=True)
            v_got = vd[q].cpu().numpy()[:T]
            y_got = torch_to_raw(yd[q], lay.dtype)
            rec = dict(slot=s, v_got=v_got, v_ref=v_ref, y_got=y_got, y_ref=y_ref, y0=y0[q], x=xs[q])
            rec["err_v"] = rel_err(v_got, v_ref)
            rec["err_y"] = rel_err(from_elt(y_got, lay.dtype), from_elt(y_ref, lay.dtype))
            out.append(rec)
            if check:
                assert not np.isnan(v_got).any(), "v has unwritten entries (slot %d)" % s
                for t in range(T):  # exact zeros where the definition says zero
                    r = self.ranks[t2a[t]] if t2a[t] >= 0 else 0
                    assert (v_got[t, r:] == 0).all()
                none = t2a < 0
                assert (y_got[none] == y0[q][none]).all(), "rows of tokens without adapter changed"
                assert rec["err_v"] <= TOL_V, "slot %d: v error %.3g" % (s, rec["err_v"])
                assert rec["err_y"] <= TOL_Y[lay.dtype], "slot %d: y error %.3g" % (s, rec["err_y"])
        return out

    def close(self):
        self.torch.cuda.synchronize()
        self.gpool.close()
        self.opool.close()
