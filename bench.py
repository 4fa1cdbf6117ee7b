#!/usr/bin/env python3
"""Benchmark of the paged multi-LoRA hot path on one MI355X.

One *step* = one decode batch through the whole path: batch translation (token -> adapter groups,
page tables to the device), shrink over all slots, expand over all slots, batch end.  Inputs
(adapter pool, activations) are resident in HBM before the timed region.  Prints ONE JSON line.

Default workload: cfg1 = Llama-7B-shaped q,k,v,o projections (4096->4096) x 32 layers = 128 slots,
bf16, 256 decode tokens, 64 resident adapters with ranks uniform in {8,16,32,64}, Zipf(1.0)
token->adapter, 64 KiB pages.  All inputs are seeded and synthetic.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

from workload import (CONFIGS, RAW_DTYPE, config_layout, draw_ranks, draw_tok2adapter, make_adapters,  # noqa: E402
                      prefill_requests, to_elt)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak
# HBM bytes per launch of the (shrink, expand) kernels measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE on the default draw of each workload, all slots per call (the profile named holds the
# commands and the counter units found on the probe kernel, whose bytes are known).  Each entry carries the
# digest of the kernel and host sources it was measured on (kernel_sources_digest below): the
# figure is reported only while the sources are still those, and null as soon as they change.
MEASURED_TRAFFIC = {
    "cfg1": dict(shrink=1.8127e9, expand=2.0986e9, profile="profiles/decode_7b_cfg1_kernels_and_hbm_traffic.md",
                 sources="6fbd2d03f7d51c49"),
    "cfg4": dict(shrink=2.3184e9, expand=2.4506e9, profile="profiles/decode_13b_layer_cfg4_kernels_and_hbm_traffic.md",
                 sources="6fbd2d03f7d51c49"),
    "cfg2": dict(shrink=0.2768e9, expand=0.4052e9, profile="profiles/prefill_cfg2_kernels_traffic_and_mfma_activity.md",
                 sources="6fbd2d03f7d51c49"),
}
METRIC = "paged LoRA shrink+expand HBM GB/s (% of peak) + tokens/s, 256-token decode"
KCLASS = ["shrink", "expand", "delta"]


def kernel_sources_digest():
    """sha256 (first 16 hex digits) over the sources that decide what the kernels do and how they are launched."""
    import hashlib
    h = hashlib.sha256()
    for name in ("plora_kernels.hip", "plora_pool.cpp", "plora_internal.h"):
        with open(os.path.join(ROOT, "paper_2512_20210_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kclass, default_draw):
    """(bytes per launch, profile) from MEASURED_TRAFFIC if it still describes the code that runs, else (None, None)."""
    rec = MEASURED_TRAFFIC.get(workload)
    if not rec or not default_draw or rec["sources"] != kernel_sources_digest():
        return None, None
    return int(rec[kclass]), rec["profile"]


def streaming_probes(P, stream, lay, ab):
    """What bare kernels reach on this GPU, for the roofline line: a plain streaming read, the same with
    a read-modify-write stream mixed in at the ratio of this workload's expand (weight bytes : y bytes),
    and one large pinned host -> device copy."""
    out = {}
    rc, ms = P.plora_probe_stream(2 << 30, 0, 64 << 10, 0, 20, stream)
    if rc == 0:
        out["read_gbs"] = round((2 << 30) / ms / 1e6, 1)
    # weights : y read (= y written) of the expand, per 4 KiB of y
    w_per_y = ab["expand_weights"] / max(ab["expand_y_read"], 1)
    w_tile = max(1, int(round(w_per_y))) * 4096
    n_tiles = max(1, (2 << 30) // (w_tile + 2 * 4096))
    rc, ms = P.plora_probe_stream(n_tiles * w_tile, n_tiles * 4096, w_tile, 4096, 20, stream)
    if rc == 0:
        out["read_plus_rmw_gbs"] = round(n_tiles * (w_tile + 2 * 4096) / ms / 1e6, 1)
        out["read_plus_rmw_mix"] = "%d KiB read : 4 KiB read-modify-write" % (w_tile // 1024)
    rc, ms = P.plora_probe_h2d(1 << 30, 3, stream)
    if rc == 0:
        out["h2d_single_pinned_copy_gbs"] = round((1 << 30) / ms / 1e6, 2)
    return out


SEED_OFFSET = 0  # --seed-offset: another draw of ranks, weights, activations and batches


def workload_params(name):
    """Ranks, scales and pool size of a named workload (all drawn from its seed)."""
    cfg = dict(CONFIGS[name])
    cfg["seed"] += SEED_OFFSET
    lay = config_layout(cfg)
    rng = np.random.default_rng(cfg["seed"])
    n_ad = cfg.get("n_adapters") or cfg["population"]
    ranks = np.asarray(cfg["ranks"], np.int32) if cfg["ranks"] else draw_ranks(rng, n_ad, cfg["rank_choices"])
    scales = [float(cfg["scale"])] * n_ad if cfg["scale"] else [16.0 / int(r) for r in ranks]
    P = cfg["page_bytes"]
    n_pages = cfg["n_pages"] or int(sum(-(-lay.adapter_bytes(int(r)) // P) for r in ranks))
    return cfg, lay, ranks, scales, P, n_pages


def draw_batch(cfg, rng, n_adapters):
    if "requests" in cfg:
        return prefill_requests(rng, cfg["requests"], cfg["len_lo"], cfg["len_hi"], np.arange(n_adapters), cfg["zipf"])[0]
    return draw_tok2adapter(rng, cfg["tokens"], np.arange(n_adapters), cfg["zipf"])


def shares_x_with_earlier_slot(lay, s):
    """--share-qkv-x: slots come in groups of four (q, k, v, o of a layer); k and v read q's x."""
    return s % 4 in (1, 2) and lay.d_in[s] == lay.d_in[s - s % 4]


def algorithmic_bytes(lay, ranks, t2a, slots, share_qkv_x=False):
    """Bytes the method itself must move for one batch over `slots` (each needed weight byte once per
    batch, x read once (once per q, k, v group with share_qkv_x), y read + written once, v written +
    read once, page-table entries and the token permutation once per slot).  Returns per-slot-summed
    dicts for shrink and expand."""
    elt = lay.elt
    has = t2a >= 0
    Tn = int(has.sum())
    uniq = np.unique(t2a[has])
    sum_r_u = int(sum(int(ranks[u]) for u in uniq))
    sum_r_t = int(sum(int(ranks[i]) for i in t2a[has]))
    shrink = expand = 0
    flops = ew = ey = 0
    for s in slots:
        di, do = lay.d_in[s], lay.d_out[s]
        meta = 4 * Tn
        x_bytes = 0 if share_qkv_x and shares_x_with_earlier_slot(lay, s) else Tn * di * elt
        shrink += sum_r_u * di * elt + x_bytes + sum_r_t * 4 + meta
        expand += sum_r_u * do * elt + 2 * Tn * do * elt + sum_r_t * 4 + meta
        ew += sum_r_u * do * elt
        ey += Tn * do * elt
        flops += 2 * sum_r_t * (di + do)
    return dict(shrink=shrink, expand=expand, total=shrink + expand, flops=flops, n_unique=len(uniq), tokens=Tn,
                expand_weights=ew, expand_y_read=ey)


class GpuWorkload:
    """Pool with all adapters resident + per-slot activation buffers on the device."""

    def __init__(self, name, workers=16, verbose=False, scatter=False):
        import torch
        import paper_2512_20210_amd as P
        self.torch, self.P, self.name = torch, P, name
        self.cfg, self.lay, self.ranks, self.scales, self.page_bytes, self.n_pages = workload_params(name)
        lay, cfg = self.lay, self.cfg
        self.n_ad = len(self.ranks)
        self.max_rank = cfg["max_rank"]
        t0 = time.perf_counter()
        self.pinned = [torch.empty(lay.adapter_elems(int(r)), dtype=torch.int16 if lay.elt == 2 else torch.float32,
                                   pin_memory=True) for r in self.ranks]
        views = [t.numpy().view(RAW_DTYPE[lay.dtype]) for t in self.pinned]
        self.blobs = make_adapters(cfg["seed"] + 1000, lay, self.ranks, outs=views, workers=workers)
        self.t_gen = time.perf_counter() - t0
        self.pool = P.PagedLoraPool(self.page_bytes, self.n_pages, lay.d_in, lay.d_out, lay.dtype, self.n_ad, self.max_rank)
        self.copy_stream = torch.cuda.Stream()
        self.stream = torch.cuda.current_stream().cuda_stream
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.tables = [self.pool.load(i, int(self.ranks[i]), self.scales[i], self.pinned[i], self.copy_stream.cuda_stream)
                       for i in range(self.n_ad)]
        self.copy_stream.synchronize()
        self.t_load = time.perf_counter() - t0
        self.stats_after_load = self.pool.stats()
        if scatter:
            # evict / reload in shuffled order twice, so that every adapter's pages are scattered
            # over the slab in short runs (the kernels then translate across many more page breaks)
            rs = np.random.default_rng(cfg["seed"] + 5)
            for rnd in range(2):
                ids = [i for i in range(self.n_ad) if i % 2 == rnd]
                rs.shuffle(ids)
                small_first = sorted(ids, key=lambda i: int(self.ranks[i]))
                for i in ids:
                    self.pool.evict(i)
                for i in (small_first if rnd == 0 else small_first[::-1]):
                    self.tables[i] = self.pool.load(i, int(self.ranks[i]), self.scales[i], self.pinned[i],
                                                    self.copy_stream.cuda_stream)
                self.copy_stream.synchronize()
        runs = sum(int((np.diff(t) != 1).sum()) + 1 for t in self.tables)
        self.mean_run_pages = sum(len(t) for t in self.tables) / runs
        if verbose:
            st = self.stats_after_load
            print("[bench] %s: %d adapters, %.2f GB in %d pages of %d KiB; generated in %.1fs; H2D %.2f GB/s wall "
                  "(%d copies, %.1f GB/s by events)" % (
                      name, self.n_ad, st["resident_bytes"] / 1e9, st["used_pages"], self.page_bytes // 1024, self.t_gen,
                      st["h2d_bytes"] / 1e9 / self.t_load, st["h2d_copies"],
                      st["h2d_bytes"] / 1e6 / max(st["h2d_ms"], 1e-9)), file=sys.stderr, flush=True)

    def alloc_activations(self, T, seed, zero_y=False, min_bytes=0, share_qkv_x=False):
        """x ~ N(0,1), y0 ~ N(0,1) per slot on the device (raw element tensors), v buffers; with
        share_qkv_x the k and v slots of a layer use the q slot's x buffer.  With
        min_bytes > 0 the whole set is replicated until it exceeds that many bytes and step() rotates
        through the replicas, so that activations cannot stay in the 256 MB last-level cache from
        one step to the next."""
        torch, lay = self.torch, self.lay
        rng = np.random.default_rng(seed)
        self.T = T
        self.share_qkv_x = share_qkv_x
        self.x, self.y, self.v = [], [], []
        # one draw per distinct width, re-used with a per-slot roll so that slots differ
        base = {}
        for s in range(lay.n_slots):
            for d in (lay.d_in[s], lay.d_out[s]):
                if d not in base:
                    base[d] = to_elt(rng.standard_normal((T, d), dtype=np.float32), lay.dtype)
        self.x_host_base, self.y_host_base = base, base
        for s in range(lay.n_slots):
            xs = np.roll(base[lay.d_in[s]], s, axis=0)
            ys = np.roll(base[lay.d_out[s]], -s - 1, axis=0)
            if share_qkv_x and shares_x_with_earlier_slot(lay, s):
                self.x.append(self.x[s - s % 4])
            else:
                self.x.append(torch.from_numpy(np.ascontiguousarray(xs).view(np.int16) if lay.elt == 2 else xs).to("cuda"))
            y = torch.from_numpy(np.ascontiguousarray(ys).view(np.int16) if lay.elt == 2 else ys).to("cuda")
            if zero_y:
                y.zero_()
            self.y.append(y)
            self.v.append(torch.empty((T, self.max_rank), dtype=torch.float32, device="cuda"))
        one = sum(t.numel() * t.element_size() for t in {id(t): t for t in self.x + self.y + self.v}.values())
        self.act_sets = [(self.x, self.y, self.v)]
        while one * len(self.act_sets) < min_bytes:
            copies = {}
            for t in self.x:  # a shared buffer stays shared in the replica
                if id(t) not in copies:
                    copies[id(t)] = t.clone()
            self.act_sets.append(([copies[id(t)] for t in self.x], [t.clone() for t in self.y], [t.clone() for t in self.v]))
        self.act_bytes, self.step_no = one, 0
        torch.cuda.synchronize()

    def host_x(self, s):
        if self.share_qkv_x and shares_x_with_earlier_slot(self.lay, s):
            s -= s % 4
        return np.roll(self.x_host_base[self.lay.d_in[s]], s, axis=0)

    def host_y0(self, s):
        return np.roll(self.y_host_base[self.lay.d_out[s]], -s - 1, axis=0)

    def step(self, t2a, slots_per_call, api="pair"):
        """api "pair": plora_shrink then plora_expand per call; "delta": plora_delta (one call, and for small
        calls one launch)."""
        pool, n = self.pool, self.lay.n_slots
        if len(t2a) > self.T:  # the library cannot see buffer sizes: never launch past the activations
            raise ValueError("batch of %d tokens but activation buffers hold %d" % (len(t2a), self.T))
        x, y, v = self.act_sets[self.step_no % len(self.act_sets)]
        self.step_no += 1
        b = pool.batch_begin(t2a, self.stream)
        for s0 in range(0, n, slots_per_call):
            s1 = min(n, s0 + slots_per_call)
            if api == "delta":
                pool.delta(b, s0, x[s0:s1], v[s0:s1], y[s0:s1], self.stream)
            else:
                pool.shrink(b, s0, x[s0:s1], v[s0:s1], self.stream)
                pool.expand(b, s0, v[s0:s1], y[s0:s1], self.stream)
        pool.batch_end(b)

    def close(self):
        self.torch.cuda.synchronize()
        self.pool.close()


def cpu_baseline(w, t2a, budget_s=15.0):
    """The oracle as it stands (fp32 accumulators, OpenMP over tokens on all host threads), timed on a
    bounded sample: whole slots of the same batch, as many as fit the time budget."""
    import oracle
    oracle.build(force=False)
    from oracle.pool import max_threads
    lay = w.lay
    threads = max_threads()
    op = oracle.OraclePool(w.page_bytes, w.n_pages, lay.d_in, lay.d_out, lay.dtype, w.n_ad, w.max_rank)
    for i in range(w.n_ad):
        op.load(i, int(w.ranks[i]), w.scales[i], w.blobs[i])
    done, t_total, bytes_total = 0, 0.0, 0
    for s in range(lay.n_slots):
        x, y = w.host_x(s), w.host_y0(s).copy()
        t0 = time.perf_counter()
        v = op.shrink(s, x, t2a, threads=threads)
        op.expand(s, v, t2a, y, threads=threads)
        t_total += time.perf_counter() - t0
        bytes_total += algorithmic_bytes(lay, w.ranks, t2a, [s], w.share_qkv_x)["total"]
        done += 1
        if t_total > budget_s or (done >= 2 and t_total / done * (done + 1) > budget_s * 1.5):
            break
    # the same loops on one thread, on the first slots only
    t1, b1, n1 = 0.0, 0, 0
    for s in range(min(2, lay.n_slots)):
        x, y = w.host_x(s), w.host_y0(s).copy()
        t0 = time.perf_counter()
        v = op.shrink(s, x, t2a, threads=1)
        op.expand(s, v, t2a, y, threads=1)
        t1 += time.perf_counter() - t0
        b1 += algorithmic_bytes(lay, w.ranks, t2a, [s], w.share_qkv_x)["total"]
        n1 += 1
    op.close()
    per_slot = t_total / done
    return dict(value=bytes_total / t_total / 1e9, unit="GB/s", cores=threads, kind="oracle",
                single_thread=dict(value=b1 / t1 / 1e9, unit="GB/s", slots=n1,
                                   tokens_per_s=len(t2a) / (t1 / n1 * lay.n_slots)),
                sample="%d of %d slots of one %d-token batch, shrink+expand, fp32 accumulators, OpenMP over tokens; "
                       "%.2f s per slot => %.1f tokens/s for the whole step" % (
                           done, lay.n_slots, len(t2a), per_slot, len(t2a) / (per_slot * lay.n_slots)),
                tokens_per_s=len(t2a) / (per_slot * lay.n_slots), seconds=t_total)


def churn_setup(name="cfg3", blobs_per_rank=8, pinned=None):
    """Pool, shared pinned blobs (blobs_per_rank distinct weight sets per rank; made unless given) and
    the request trace (windows; long enough for the configured number of load / evict events)."""
    import torch
    import paper_2512_20210_amd as P
    from workload import churn_trace, make_adapter
    cfg, lay, ranks, scales, page_bytes, n_pages = workload_params(name)
    pop = cfg["population"]
    rng = np.random.default_rng(cfg["seed"] + 1000)
    make = pinned is None
    pinned = {} if make else pinned
    for r in sorted(set(int(x) for x in ranks)) if make else ():
        for k in range(blobs_per_rank):
            t = torch.empty(lay.adapter_elems(r), dtype=torch.int16, pin_memory=True)
            make_adapter(rng, lay, r, out=t.numpy().view(np.uint16))
            pinned[(r, k)] = t
    pool = P.PagedLoraPool(page_bytes, n_pages, lay.d_in, lay.d_out, lay.dtype, pop, cfg["max_rank"])
    trace = churn_trace(np.random.default_rng(cfg["seed"] + 1), cfg.get("max_requests", cfg["n_events"]), pop, cfg["zipf"],
                        cfg["window"], cfg["burst_prob"], cfg["burst_mult"])
    return cfg, lay, ranks, scales, pool, pinned, trace


def _churn_pass(cfg, lay, ranks, scales, pool, pinned, trace, quality, stop_on="events"):
    """One pass over the churn trace, driven by the library's residency policy (plora_manager_*).  quality
    None: adapters are loaded on demand only; a number: threshold prefetching on a synthetic prediction
    of that quality before every window; "lstm": on the library's predictor, which learns online from
    the windows it has seen.  stop_on "events": the pass ends with the window in which the number of
    loads + evictions reaches cfg["n_events"]; "requests": after cfg["n_events"] requests."""
    import torch
    import paper_2512_20210_amd as P
    from workload import SyntheticPredictor, zipf_probs
    pop, T = cfg["population"], cfg["tokens"]
    k_blobs = len(pinned) // len(set(int(x) for x in ranks))
    copy_stream, prefetch_stream = torch.cuda.Stream(), torch.cuda.Stream()
    stream = torch.cuda.current_stream().cuda_stream
    popularity = zipf_probs(pop, cfg["zipf"])
    mgr = P.ResidencyManager(pool, ranks, scales, lambda i: pinned[(int(ranks[i]), i % k_blobs)],
                             copy_stream=copy_stream.cuda_stream, prefetch_stream=prefetch_stream.cuda_stream)
    mgr.set_prediction(popularity / popularity.max())
    if quality == "lstm":
        pred = P.LstmPredictor(pop, window=cfg.get("lstm_window", 8), hidden=64, layers=2, replay=10000, batch=64,
                               lr=cfg.get("lstm_lr", 1e-3), seed=cfg["seed"] + 13, train_steps=cfg.get("lstm_steps", 1),
                               threads=min(16, os.cpu_count() or 1))
    else:
        pred = SyntheticPredictor(pop, popularity, quality, seed=cfg["seed"] + 11) if quality is not None else None
    per_window = []       # (requests, cold starts, |predicted & requested|, |predicted|, |requested|) per window
    pred_s = 0.0
    rng = np.random.default_rng(cfg["seed"] + 7)
    base = {d: to_elt(rng.standard_normal((T, d), dtype=np.float32), lay.dtype).view(np.int16) for d in set(lay.d_in) | set(lay.d_out)}
    x = [torch.from_numpy(np.roll(base[d], s, axis=0)).cuda() for s, d in enumerate(lay.d_in)]
    y = [torch.from_numpy(np.roll(base[d], -s - 1, axis=0)).cuda() for s, d in enumerate(lay.d_out)]
    v = [torch.empty((T, cfg["max_rank"]), dtype=torch.float32, device="cuda") for _ in lay.d_in]
    slots = list(range(lay.n_slots))
    pool.profile(True)
    events = batches = 0
    kbytes = 0
    pending, ttr_ms = {}, []   # cold misses whose copy is still running -> host time of the request
    prefetched_ready = prefetched_first_use = 0
    cold = 0

    def poll():
        now = time.perf_counter()
        for a in list(pending):
            if not mgr.state(a) & 1:    # became ready and was evicted again between two polls
                del pending[a]
            elif pool.ready(a):
                ttr_ms.append((now - pending.pop(a)) * 1e3)

    def done():
        if stop_on == "requests":
            return events >= cfg["n_events"]
        st = pool.stats()
        return st["loads"] + st["evictions"] >= cfg["n_events"]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for win in trace:
        cold0, ev0 = cold, events
        hit_pred = n_pred = 0
        if pred is not None:  # between two decode batches: the copies run beside the next batch's kernels
            tp = time.perf_counter()
            p_hat = pred.predict(win)
            pred_s += time.perf_counter() - tp
            flagged = set(np.nonzero(p_hat > mgr.theta)[0].tolist())
            hit_pred, n_pred = len(flagged & set(int(a) for a in win)), len(flagged)
            mgr.prefetch(p_hat)
        for aid in win:
            aid = int(aid)
            if mgr.state(aid) & 2:
                prefetched_first_use += 1
                prefetched_ready += bool(pool.ready(aid))
            if not mgr.request(aid):
                cold += 1
                if mgr.state(aid) & 1:
                    pending[aid] = time.perf_counter()
            if pending:
                poll()
            events += 1
            if stop_on == "requests" and events >= cfg["n_events"]:
                break
        res = mgr.residents()
        p = popularity[res] / popularity[res].sum()
        t2a = res[rng.choice(len(res), size=T, p=p)].astype(np.int32)
        b = pool.batch_begin(t2a, stream)
        pool.shrink(b, 0, x, v, stream)
        pool.expand(b, 0, v, y, stream)
        pool.batch_end(b)
        kbytes += algorithmic_bytes(lay, ranks, t2a, slots)["total"]
        batches += 1
        per_window.append((events - ev0, cold - cold0, hit_pred, n_pred, len(set(int(a) for a in win))))
        if done():
            break
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    poll()
    kms, kn = pool.profile_read()
    st, ms = pool.stats(), mgr.stats()
    n_util = max(ms["util_samples"], 1)
    out = {
        "prediction_quality": quality, "requests": events, "load_plus_evict_events": st["loads"] + st["evictions"],
        "decode_batches": batches, "wall_s": round(wall, 3),
        "page_util_avg": round(ms["page_util_sum"] / n_util, 4), "page_util_min": round(ms["page_util_min"], 4),
        "byte_util_avg": round(ms["byte_util_sum"] / n_util, 4), "byte_util_min": round(ms["byte_util_min"], 4),
        "hit_rate": round(ms["hits"] / max(1, ms["hits"] + ms["misses"]), 4),
        "cold_start_rate": round(ms["misses"] / max(1, events), 4),
        "cold_time_to_ready_ms_mean": round(float(np.mean(ttr_ms)), 3) if ttr_ms else None,
        "cold_time_to_ready_ms_p95": round(float(np.percentile(ttr_ms, 95)), 3) if ttr_ms else None,
        "prefetch_loads": ms["prefetch_loads"], "useful_prefetches": ms["useful_prefetches"],
        "wasted_prefetches": ms["wasted_prefetches"],
        "prefetched_ready_at_first_use": round(prefetched_ready / max(1, prefetched_first_use), 4) if pred is not None else None,
        "loads": st["loads"], "evictions": st["evictions"],
        "skipped_busy_victims": ms["skipped_busy"], "host_waits_for_a_busy_victim": ms["waited_for_busy"], "failed_loads": ms["failed_loads"],
        "h2d_gb": round(st["h2d_bytes"] / 1e9, 2), "h2d_copies": st["h2d_copies"],
        "h2d_gbs_copy_time": round(st["h2d_bytes"] / 1e6 / max(st["h2d_ms"], 1e-9), 2),
        "h2d_gbs_wall": round(st["h2d_bytes"] / 1e9 / wall, 2),
        "decode_kernel_gbs": round(kbytes / 1e6 / max(sum(kms), 1e-9), 1),
        "decode_kernel_ms_per_batch": round(sum(kms) / max(batches, 1), 4),
        "resident_adapters_end": st["resident_adapters"],
    }
    # the last quarter of the windows on its own: an online predictor has had time to learn by then
    tail = np.array(per_window[-max(1, len(per_window) // 4):], dtype=np.float64).sum(0)
    out["last_quarter"] = {"cold_start_rate": round(tail[1] / max(tail[0], 1), 4),
                           "prediction_recall": round(tail[2] / max(tail[4], 1), 4) if pred is not None else None,
                           "prediction_precision": round(tail[2] / max(tail[3], 1), 4) if pred is not None else None}
    if pred is not None:
        out["predictor_ms_per_window"] = round(pred_s / max(len(per_window), 1) * 1e3, 3)
    if quality == "lstm":
        pred.close()
    mgr.close()
    return out


def run_load_study(args):
    """H2D rate of plora_load_adapter into fragmented pools, direct (one copy per run of consecutive
    pages) against staged (one copy + scatter kernel), and direct again after plora_compact has made the
    free pages one range: cfg3's one-layer slots and 64 KiB pages, free space made of holes of h pages,
    32 rank-64 adapters (4 MiB = 64 pages each) loaded back to back."""
    import torch
    import paper_2512_20210_amd as P
    from workload import make_adapter
    cfg, lay, _, _, page_bytes, _ = workload_params("cfg3")
    rng = np.random.default_rng(cfg["seed"] + 2000)
    big_rank, n_big = 64, 32
    big_pages = lay.adapter_elems(big_rank) * 2 // page_bytes
    unit_rank = page_bytes // (lay.adapter_elems(1) * 2)          # rank whose blob is exactly one page
    assert unit_rank * lay.adapter_elems(1) * 2 == page_bytes

    def pinned_blob(r):
        t = torch.empty(lay.adapter_elems(r), dtype=torch.int16, pin_memory=True)
        make_adapter(rng, lay, r, out=t.numpy().view(np.uint16))
        return t
    big = [pinned_blob(big_rank) for _ in range(4)]
    copy_stream = torch.cuda.Stream()
    rows = []
    for hole in (1, 2, 4, 16, 32, 0):   # 0: an empty pool, every adapter lands on consecutive pages
        n_fill = 0 if hole == 0 else 2 * (n_big * big_pages // hole)
        n_pages = n_fill * max(hole, 1) + n_big * big_pages
        pool = P.PagedLoraPool(page_bytes, n_pages, lay.d_in, lay.d_out, lay.dtype, n_fill + n_big, 128)
        if hole:
            filler = pinned_blob(hole * unit_rank)
            for i in range(n_fill):
                pool.load(i, hole * unit_rank, 1.0, filler, copy_stream.cuda_stream)
            torch.cuda.synchronize()
            for i in range(0, n_fill, 2):
                pool.evict(i)
        row = {"hole_pages": hole or None, "runs_per_adapter": None}
        for mode in ("direct", "staged", "direct", "staged"):   # the second round is the one reported
            pool.set_option("staging_bytes", lay.adapter_elems(big_rank) * 2 if mode == "staged" else 0)
            c0 = pool.stats()["h2d_copies"]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(n_big):
                pool.load(n_fill + k, big_rank, 0.25, big[k % len(big)], copy_stream.cuda_stream)
            t_issue = time.perf_counter() - t0
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            st = pool.stats()
            row["runs_per_adapter"] = (st["h2d_copies"] - c0) / n_big if mode == "direct" else row["runs_per_adapter"]
            row[mode + "_gbs"] = round(n_big * lay.adapter_elems(big_rank) * 2 / dt / 1e9, 2)
            row[mode + "_host_issue_ms"] = round(t_issue * 1e3, 2)
            for k in range(n_big):
                pool.evict(n_fill + k)
        row["staged_loads"] = pool.stats()["staged_loads"]
        if hole:
            # the same pool after plora_compact: the fillers slide down, the free pages become one range
            pool.set_option("staging_bytes", 0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            pages, adapters = pool.compact(copy_stream.cuda_stream)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            row["compaction"] = {"pages_moved": pages, "adapters_moved": adapters, "ms": round(dt * 1e3, 2),
                                 "moved_gbs": round(pages * page_bytes / dt / 1e9, 2)}
            for rep in range(2):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for k in range(n_big):
                    pool.load(n_fill + k, big_rank, 0.25, big[k % len(big)], copy_stream.cuda_stream)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                row["direct_after_compaction_gbs"] = round(n_big * lay.adapter_elems(big_rank) * 2 / dt / 1e9, 2)
                for k in range(n_big):
                    pool.evict(n_fill + k)
        rows.append(row)
        pool.close()
    print(json.dumps({"metric": "H2D GB/s of adapter loads into fragmented pools: direct, staged, direct after compaction", "workload": "load_study",
                      "adapter_bytes": lay.adapter_elems(big_rank) * 2, "adapters": n_big, "page_bytes": page_bytes, "rows": rows}))


def run_churn_periodic(args):
    """cfg3p: the churn workload with a recurring request pattern (timer-like adapters on top of a Zipf
    background) and a pool that holds a third of the adapters in play: loads on demand, the library's
    LSTM predictor learning online, and a synthetic prediction of quality 0.86 for comparison."""
    from workload import periodic_trace
    out = {"metric": "cold starts under a recurring request pattern: on demand vs LSTM-predicted prefetch",
           "workload": "cfg3p", "passes": []}
    pinned = None
    for quality in (None, "lstm", 0.86):
        cfg, lay, ranks, scales, pool, pinned, _ = churn_setup("cfg3p", pinned=pinned)
        trace = periodic_trace(np.random.default_rng(cfg["seed"] + 1), cfg["n_events"] // cfg["window"], cfg["population"],
                               cfg["zipf"], cfg["window"], cfg["n_periodic"], cfg["periods"])
        out["passes"].append(_churn_pass(cfg, lay, ranks, scales, pool, pinned, trace, quality, stop_on="requests"))
        pool.close()
    print(json.dumps(out))


def run_churn(args):
    """cfg3: load/evict churn interleaved with decode batches until 10,000 loads + evictions have
    happened; utilisation, H2D and kernel rates, with loads on demand only and with threshold
    prefetching on a synthetic prediction (direct and staged copies); then the same for the reading in
    which an adapter covers all 32 layers (cfg3L: 8 .. 256 MiB per adapter, about two dozen resident)."""
    import paper_2512_20210_amd as P
    out = {"metric": "pool utilisation under churn + H2D prefetch GB/s + decode kernel GB/s + cold starts",
           "workload": "cfg3", "passes": [], "passes_32_layer_adapters": []}
    rc, ms = P.plora_probe_h2d(1 << 30, 3, None)
    if rc == 0:
        out["h2d_single_pinned_copy_gbs"] = round((1 << 30) / ms / 1e6, 2)
    pinned = None
    for quality, staged in ((None, False), (0.86, False), (0.86, True)):
        cfg, lay, ranks, scales, pool, pinned, trace = churn_setup("cfg3", pinned=pinned)
        if staged:  # every blob of two or more runs of pages goes through a staging buffer
            pool.set_option("staging_bytes", lay.adapter_elems(cfg["max_rank"]) * 2)
        res = _churn_pass(cfg, lay, ranks, scales, pool, pinned, trace, quality)
        res["staged_loads"] = pool.stats()["staged_loads"]
        out["passes"].append(res)
        pool.close()
    pinned = None
    for quality in (None, 0.86):
        cfg, lay, ranks, scales, pool, pinned, trace = churn_setup("cfg3L", blobs_per_rank=1, pinned=pinned)
        out["passes_32_layer_adapters"].append(_churn_pass(cfg, lay, ranks, scales, pool, pinned, trace, quality))
        pool.close()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg1", choices=["cfg0", "cfg1", "cfg2", "cfg2x8", "cfg3", "cfg3p", "cfg4", "cfg5", "load_study"])
    ap.add_argument("--slots-per-call", type=int, default=0, help="slots per plora_shrink/plora_expand call (0 = all)")
    ap.add_argument("--mfma-min-tokens", type=int, default=-1, help="plain token threshold of the matrix-core items in shrink (default: the library's work-based rule)")
    ap.add_argument("--mfma-min-tokens-expand", type=int, default=-1, help="the same for expand")
    ap.add_argument("--xcd-remap", type=int, default=-1)
    ap.add_argument("--coop-max-workgroups", type=int, default=-1,
                    help="calls of at most this many workgroups use the cooperative kernels (library defaults 192 for "
                         "shrink, 2500 for expand; 0 = never)")
    ap.add_argument("--api", default="pair", choices=["pair", "delta"], help="plora_shrink + plora_expand per call, or plora_delta")
    ap.add_argument("--opt", action="append", default=[], help="key=value passed to plora_pool_set_option (repeatable)")
    ap.add_argument("--no-probes", action="store_true", help="skip the streaming / copy probes")
    ap.add_argument("--no-per-layer", action="store_true", help="skip the leg that repeats the steps with one call per layer (4 slots)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--share-qkv-x", action="store_true", help="k and v slots of a layer read the q slot's x buffer (as in a transformer layer); x is then counted once per group")
    ap.add_argument("--same-batch", action="store_true", help="reuse one token->adapter draw for every step")
    ap.add_argument("--scatter", action="store_true", help="evict and reload adapters so that their pages are scattered")
    ap.add_argument("--seed-offset", type=int, default=0, help="added to the workload's seed: another draw of ranks, weights and batches")
    ap.add_argument("--verbose", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the path has no multi-GPU part", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    global SEED_OFFSET
    SEED_OFFSET = args.seed_offset
    if args.workload == "cfg3":
        run_churn(args)
        return
    if args.workload == "cfg3p":
        run_churn_periodic(args)
        return
    if args.workload == "load_study":
        run_load_study(args)
        return

    w = GpuWorkload(args.workload, verbose=args.verbose, scatter=args.scatter)
    cfg, lay = w.cfg, w.lay
    if args.coop_max_workgroups >= 0:
        w.pool.set_option("coop_max_workgroups_shrink", args.coop_max_workgroups)
        w.pool.set_option("coop_max_workgroups_expand", args.coop_max_workgroups)
    if args.mfma_min_tokens >= 0:   # a plain token threshold: the work condition is switched off
        w.pool.set_option("mfma_min_tokens", args.mfma_min_tokens)
        w.pool.set_option("mfma_min_work", 1 << 30)
    if args.mfma_min_tokens_expand >= 0:
        w.pool.set_option("mfma_min_tokens_expand", args.mfma_min_tokens_expand)
        w.pool.set_option("mfma_min_work_expand", 1 << 30)
    if args.xcd_remap >= 0:
        w.pool.set_option("xcd_remap", args.xcd_remap)
    for kv in args.opt:
        key, val = kv.split("=")
        w.pool.set_option(key, int(val))
    rng = np.random.default_rng(cfg["seed"] + 7)
    n_draws = 1 if args.same_batch else args.steps + args.warmup
    batches = [draw_batch(cfg, rng, w.n_ad) for _ in range(n_draws)]
    T = max(len(b) for b in batches)
    w.alloc_activations(T, cfg["seed"] + 9, min_bytes=768 << 20, share_qkv_x=args.share_qkv_x)
    spc = args.slots_per_call or lay.n_slots
    all_slots = list(range(lay.n_slots))

    for i in range(args.warmup):
        w.step(batches[i % n_draws], spc, args.api)
    torch.cuda.synchronize()
    if not args.no_kernel_events:
        w.pool.profile(True)
    timed = [batches[(args.warmup + i) % n_draws] for i in range(args.steps)]
    t0 = time.perf_counter()
    for t2a in timed:
        w.step(t2a, spc, args.api)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    kms, kn = ([0.0] * 3, [0] * 3)
    if not args.no_kernel_events:
        w.pool.profile(False)
        kms, kn = w.pool.profile_read()

    ab = [algorithmic_bytes(lay, w.ranks, t2a, all_slots, args.share_qkv_x) for t2a in timed]
    bytes_total = sum(a["total"] for a in ab)
    tokens_total = sum(len(t2a) for t2a in timed)
    gbs = bytes_total / elapsed / 1e9

    # dominant kernel: the class with the largest summed duration; its algorithmic bytes per launch
    # are the weights of its adapter groups plus the activations of their tokens (split by path)
    roof = None
    if not args.no_kernel_events and sum(kn):
        dom = int(np.argmax(kms))
        kb = sum(a[("shrink", "expand", "total")[dom]] for a in ab)
        avg_ms = kms[dom] / kn[dom]
        per_launch = kb / kn[dom]
        ach = per_launch / (avg_ms * 1e-3) / 1e9
        default_draw = spc == lay.n_slots and SEED_OFFSET == 0 and not args.share_qkv_x
        traffic, traffic_profile = measured_traffic(args.workload, KCLASS[dom], default_draw and dom < 2)
        roof = dict(bound="hbm", kernel=KCLASS[dom], achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(ach / HBM_PEAK_GBS, 4), traffic=traffic, traffic_profile=traffic_profile,
                    kernel_sources=kernel_sources_digest(), avg_launch_ms=round(avg_ms, 5),
                    launches=int(kn[dom]), algorithmic_bytes_per_launch=int(per_launch),
                    all_kernels_ms_per_step={KCLASS[k]: round(kms[k] / args.steps, 5) for k in range(3) if kn[k]})

    out = {
        "metric": METRIC, "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": {0: "f16", 1: "bf16", 2: "f32"}[lay.dtype],
        "data": "synthetic",
        "config": {"workload": args.workload, "slots": lay.n_slots, "tokens": int(T), "adapters": int(w.n_ad),
                   "page_bytes": int(w.page_bytes), "pool_pages": int(w.n_pages), "slots_per_call": int(spc), "entry_points": args.api, "seed": int(cfg["seed"]), "share_qkv_x": bool(args.share_qkv_x),
                   "mean_unique_adapters": round(float(np.mean([a["n_unique"] for a in ab])), 1),
                   "mean_run_of_consecutive_pages": round(w.mean_run_pages, 1), "activation_sets": len(w.act_sets), "activation_bytes_per_set": int(w.act_bytes)},
        "tokens_per_s": round(tokens_total / elapsed, 1),
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "algorithmic_bytes_per_step": int(bytes_total / args.steps),
        "algorithmic_bytes_per_step_by_kernel": {"shrink": int(sum(a["shrink"] for a in ab) / args.steps),
                                                 "expand": int(sum(a["expand"] for a in ab) / args.steps)},
        "gflop_per_step": round(sum(a["flops"] for a in ab) / args.steps / 1e9, 2),
        "h2d_prefetch_gbs": round(w.stats_after_load["h2d_bytes"] / 1e9 / w.t_load, 2),
        "pool_page_util": round(w.stats_after_load["used_pages"] / w.stats_after_load["n_pages"], 4),
        "roofline": roof,
    }
    if not args.no_kernel_events:
        # The timed steps above carry a pair of timing events on every kernel dispatch (the roofline figures need
        # them), and a dispatch with events costs the queue a few microseconds: the same steps without them.
        n = min(args.steps, 200)
        t0 = time.perf_counter()
        for i in range(n):
            w.step(timed[i], spc, args.api)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        bn = sum(a["total"] for a in ab[:n])
        out["without_kernel_events"] = {"steps": n, "ms_per_step": round(dt / n * 1e3, 4), "value": round(bn / dt / 1e9, 1),
                                        "unit": "GB/s", "pct_of_hbm_peak": round(100.0 * bn / dt / 1e9 / HBM_PEAK_GBS, 2),
                                        "tokens_per_s": round(sum(len(t) for t in timed[:n]) / dt, 1)}
    if not args.no_per_layer:
        # the same steps as a layer-by-layer decoder has to issue them: one call per layer (4 slots)
        if lay.n_slots > 4 and lay.n_slots % 4 == 0 and spc == lay.n_slots:
            n = min(args.steps, 200)
            for i in range(10):
                w.step(timed[i % len(timed)], 4, "delta")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(n):
                w.step(timed[i % len(timed)], 4, "delta")
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            b4 = sum(ab[i % len(timed)]["total"] for i in range(n))
            out["per_layer_calls"] = {"slots_per_call": 4, "entry_points": "delta", "steps": n, "ms_per_step": round(dt / n * 1e3, 4),
                                      "value": round(b4 / dt / 1e9, 1), "unit": "GB/s",
                                      "pct_of_hbm_peak": round(100.0 * b4 / dt / 1e9 / HBM_PEAK_GBS, 2),
                                      "tokens_per_s": round(sum(len(timed[i % len(timed)]) for i in range(n)) / dt, 1)}
    if not args.no_probes:
        probes = streaming_probes(w.P, w.stream, lay, ab[0])
        out["streaming_roof"] = probes
        if probes.get("read_gbs"):
            out["pct_of_streaming_roof"] = round(100.0 * gbs / probes["read_gbs"], 2)
        if roof is not None and probes.get("read_plus_rmw_gbs"):
            roof["vs_probe_of_same_mix"] = round(roof["achieved"] / (probes["read_plus_rmw_gbs"] if roof["kernel"] == "expand" else probes["read_gbs"]), 4)
        if probes.get("h2d_single_pinned_copy_gbs"):
            out["h2d_pct_of_single_pinned_copy"] = round(100.0 * out["h2d_prefetch_gbs"] / probes["h2d_single_pinned_copy_gbs"], 1)
    # The loads above were the first use of the slab and of the pinned blobs.  What a pool that has been running
    # for a while sees: every adapter evicted and loaded again, same stream, same placement.
    torch.cuda.synchronize()
    for i in range(w.n_ad):
        w.pool.evict(i)
    t0 = time.perf_counter()
    for i in range(w.n_ad):
        w.pool.load(i, int(w.ranks[i]), w.scales[i], w.pinned[i], w.copy_stream.cuda_stream)
    w.copy_stream.synchronize()
    out["h2d_reload_gbs"] = round(w.stats_after_load["h2d_bytes"] / 1e9 / (time.perf_counter() - t0), 2)
    if out.get("streaming_roof", {}).get("h2d_single_pinned_copy_gbs"):
        out["h2d_reload_pct_of_single_pinned_copy"] = round(100.0 * out["h2d_reload_gbs"] / out["streaming_roof"]["h2d_single_pinned_copy_gbs"], 1)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, timed[0])
    w.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
