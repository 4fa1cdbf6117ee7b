"""The named workloads (shapes only; every draw is seeded)."""
from .gen import DT_BF16, DT_F16, Layout

BASE_SEED = 20251220  # config k uses BASE_SEED + k

KIB = 1024

CONFIGS = {
    # one 1024->1024 fp16 linear, 16 decode tokens, 4 adapters of ranks (8,16,8,16), uniform
    # token->adapter draw, scale 2, 16 KiB pages, 64 pages
    "cfg0": dict(seed=BASE_SEED + 0, dtype=DT_F16, slots=[(1024, 1024)], tokens=16, n_adapters=4,
                 ranks=[8, 16, 8, 16], rank_choices=None, zipf=None, scale=2.0, page_bytes=16 * KIB,
                 n_pages=64, max_rank=16),
    # Llama-7B-shaped attention projections q,k,v,o (4096->4096) x 32 layers, bf16, 256 decode
    # tokens, 64 resident adapters with ranks uniform in {8,16,32,64}, Zipf(1.0), 64 KiB pages
    "cfg1": dict(seed=BASE_SEED + 1, dtype=DT_BF16, slots=[(4096, 4096)] * 128, tokens=256, n_adapters=64,
                 ranks=None, rank_choices=[8, 16, 32, 64], zipf=1.0, scale=None, page_bytes=64 * KIB,
                 n_pages=None, max_rank=64),
    # prefill: 32 requests of length U[64,256], hidden 4096, bf16, 128 adapters with ranks uniform
    # in {8,...,128}, Zipf(1.2) request->adapter; q,k,v,o of one layer
    "cfg2": dict(seed=BASE_SEED + 2, dtype=DT_BF16, slots=[(4096, 4096)] * 4, requests=32, len_lo=64,
                 len_hi=256, n_adapters=128, ranks=None, rank_choices=[8, 16, 32, 64, 128], zipf=1.2,
                 scale=None, page_bytes=64 * KIB, n_pages=None, max_rank=128),
    # the same prefill batch over 8 layers (32 slots): shows the kernels with ample parallelism
    "cfg2x8": dict(seed=BASE_SEED + 2, dtype=DT_BF16, slots=[(4096, 4096)] * 32, requests=32, len_lo=64,
                   len_hi=256, n_adapters=128, ranks=None, rank_choices=[8, 16, 32, 64, 128], zipf=1.2,
                   scale=None, page_bytes=64 * KIB, n_pages=None, max_rank=128),
    # churn: 2 GiB pool of 64 KiB pages driven until 10,000 load / evict events have happened, by
    # requests over a population of adapters with ranks in {4,...,128}, Zipf(1.0) popularity, bursts
    # (x8 for 10% of windows), interleaved with 512-token bf16 decode batches at hidden 4096
    # (q,k,v,o of one layer); max_requests bounds the trace that is drawn
    "cfg3": dict(seed=BASE_SEED + 3, dtype=DT_BF16, slots=[(4096, 4096)] * 4, tokens=512, population=4096,
                 ranks=None, rank_choices=[4, 8, 16, 32, 64, 128], zipf=1.0, scale=None,
                 page_bytes=64 * KIB, n_pages=32768, max_rank=128, n_events=10000, max_requests=80000, window=100,
                 burst_prob=0.1, burst_mult=8),
    # the same with adapters that cover all 32 layers (128 slots): 8 .. 256 MiB each, two dozen of a
    # population of 256 fit the 2 GiB pool (one rank-128 adapter is an eighth of it)
    "cfg3L": dict(seed=BASE_SEED + 3, dtype=DT_BF16, slots=[(4096, 4096)] * 128, tokens=512, population=256,
                  ranks=None, rank_choices=[4, 8, 16, 32, 64, 128], zipf=1.0, scale=None,
                  page_bytes=64 * KIB, n_pages=32768, max_rank=128, n_events=10000, max_requests=80000, window=100,
                  burst_prob=0.1, burst_mult=8),
    # cfg3 with a recurring request pattern (300 timer-like adapters with periods of 2 .. 12 windows on a
    # Zipf background) and a pool of a fifth of cfg3's size, so that long-period adapters are evicted
    # between two of their windows; for the traffic predictor (Sec. III-A)
    "cfg3p": dict(seed=BASE_SEED + 6, dtype=DT_BF16, slots=[(4096, 4096)] * 4, tokens=512, population=4096,
                  ranks=None, rank_choices=[4, 8, 16, 32, 64, 128], zipf=1.0, scale=None,
                  page_bytes=64 * KIB, n_pages=6400, max_rank=128, n_events=80000, window=100,
                  burst_prob=0.0, burst_mult=1, n_periodic=300, periods=(2, 3, 4, 6, 8, 12),
                  lstm_window=12, lstm_lr=3e-3, lstm_steps=4),
    # one Llama-13B-shaped layer: q,k,v,o 5120->5120, up 5120->13824, down 13824->5120, bf16,
    # 1024-token decode batch over 1000 resident adapters, ranks uniform in {16,...,128}, Zipf(0.8),
    # 128 KiB pages, pool sized to the whole adapter set
    "cfg4": dict(seed=BASE_SEED + 4, dtype=DT_BF16,
                 slots=[(5120, 5120)] * 4 + [(5120, 13824), (13824, 5120)], tokens=1024, n_adapters=1000,
                 ranks=None, rank_choices=[16, 32, 64, 128], zipf=0.8, scale=None, page_bytes=128 * KIB,
                 n_pages=None, max_rank=128),
    # Mistral-7B-shaped attention projections (grouped-query attention: q, o 4096->4096, k, v 4096->1024)
    # x 32 layers; everything else as cfg1 (the second model of Sec. V-A)
    "cfg5": dict(seed=BASE_SEED + 5, dtype=DT_BF16, slots=[(4096, 4096), (4096, 1024), (4096, 1024), (4096, 4096)] * 32,
                 tokens=256, n_adapters=64, ranks=None, rank_choices=[8, 16, 32, 64], zipf=1.0, scale=None,
                 page_bytes=64 * KIB, n_pages=None, max_rank=64),
}


def config_layout(cfg):
    return Layout(tuple(s[0] for s in cfg["slots"]), tuple(s[1] for s in cfg["slots"]), cfg["dtype"])
