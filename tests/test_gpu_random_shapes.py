"""GPU parity on seeded random shapes: layouts, ranks, page sizes, batch compositions and dispatch
thresholds drawn at random (every case printed before it runs), group sizes placed on the tile
boundaries of the kernels (4 / 5 tokens per vector-ALU item, 16 / 17 per column-split item, 32 / 33
per matrix-core shrink tile, 64 / 65 per panel, 128 / 129 per block of a large group)."""
import numpy as np
import pytest

from workload import DT_BF16, DT_F16, DT_F32, Layout
from helpers import Case

pytestmark = pytest.mark.gpu

EDGES = (1, 2, 4, 5, 15, 16, 17, 31, 32, 33, 48, 63, 64, 65, 100, 127, 128, 129, 200)


@pytest.mark.parametrize("seed", list(range(40)))
def test_random_case(oracle_mod, seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = [DT_BF16, DT_BF16, DT_F16, DT_F32][seed % 4]
    n_slots = int(rng.integers(1, 4))
    dims = lambda: tuple(int(8 * rng.integers(1, 180)) for _ in range(n_slots))
    lay = Layout(dims(), dims(), dtype)
    n_ad = int(rng.integers(2, 7))
    ranks = [int(rng.choice([1, 3, 8, 16, 17, 32, 40, 64, 100, 128])) for _ in range(n_ad)]
    page = int(rng.choice([4096, 16384, 65536, 1 << 20]))
    elt = 4 if dtype == DT_F32 else 2
    C = sum(lay.d_in) + sum(lay.d_out)
    need = sum(-(-(r * elt * C) // page) for r in ranks)
    groups = [int(rng.choice(EDGES)) for _ in range(n_ad)]
    t2a = np.concatenate([np.full(n, a, np.int32) for a, n in enumerate(groups)] + [np.full(int(rng.integers(0, 6)), -1, np.int32)])
    rng.shuffle(t2a)
    mfma = int(rng.choice([0, 1, 2, 6, 16]))
    print("seed", seed, "dtype", dtype, "d_in", lay.d_in, "d_out", lay.d_out, "ranks", ranks, "page", page,
          "groups", groups, "mfma_min_tokens", mfma, flush=True)
    order = rng.permutation(n_ad).tolist()
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], page, need + 3, seed=seed, max_rank=max(ranks) + int(rng.integers(0, 3)),
                load_order=order, mfma_min_tokens=mfma)
    if seed % 3 == 0:  # scatter the pages of one adapter
        case.evict(order[0])
        case.load(order[0])
    if seed % 2:
        case.gpool.set_option("slot_major", int(rng.integers(0, 2)))
        case.gpool.set_option("xcd_remap", int(rng.integers(0, 2)))
    out = case.run(t2a, seed=seed)
    print("   err_v", ["%.2g" % o["err_v"] for o in out], "err_y", ["%.2g" % o["err_y"] for o in out], flush=True)
    case.close()
