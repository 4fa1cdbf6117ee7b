"""plora_delta as one launch (option "fused_max_tasks"): shrink and expand tasks of a small call run by one
persistent grid, an expand task waiting, bounded, for its slot's shrink tasks.

* the results are those of plora_shrink + plora_expand, bit for bit, and match the oracle (Case.run does the
  same on every parity case; here several calls in a row reuse one batch's counters, as per-layer calls do);
* with the wait cut to a single poll from the host, the launch still ends: tasks that found their slot
  unfinished are given up and counted (plora_stats.fused_timeouts), and the next ordinary call is right;
* a stream under graph capture takes the two launches (a replay would reuse the call's counter targets).
"""
import numpy as np
import pytest

from workload import DT_BF16, DT_F16, Layout, draw_tok2adapter, from_elt, make_act
from helpers import TOL_Y, Case, raw_to_torch, rel_err, torch_to_raw

pytestmark = pytest.mark.gpu


def _setup(oracle_mod, dtype=DT_BF16):
    lay = Layout((1024, 520, 256, 1024, 512, 512), (1024, 264, 1544, 512, 512, 1024), dtype)
    ranks = [8, 16, 3, 40, 64, 24, 32, 5]
    case = Case(oracle_mod, lay, ranks, [16.0 / r for r in ranks], 16384, 1024, seed=47)
    return case, lay, ranks


@pytest.mark.parametrize("dtype,coop", [(DT_BF16, 0), (DT_BF16, 1 << 30), (DT_F16, 0)])
def test_one_launch_equals_two_launches_over_many_calls_on_one_batch(oracle_mod, dtype, coop):
    import torch
    case, lay, ranks = _setup(oracle_mod, dtype)
    pool = case.gpool
    pool.set_option("coop_max_workgroups_shrink", coop)
    pool.set_option("coop_max_workgroups_expand", coop)
    rng = np.random.default_rng(5)
    T = 200
    t2a = draw_tok2adapter(rng, T, np.arange(len(ranks)), s=1.0, none_frac=0.1)
    xs = [make_act(rng, T, d, lay.dtype) for d in lay.d_in]
    y0 = [make_act(rng, T, d, lay.dtype) for d in lay.d_out]
    xd = [raw_to_torch(a, "cuda") for a in xs]
    y_two = [raw_to_torch(a, "cuda") for a in y0]
    y_one = [raw_to_torch(a, "cuda") for a in y0]
    v_two = [torch.full((T, case.max_rank), float("nan"), device="cuda") for _ in xs]
    v_one = [torch.full((T, case.max_rank), float("nan"), device="cuda") for _ in xs]
    batch = pool.batch_begin(t2a, case.stream)
    calls = ((0, 1), (1, 3), (3, 6), (0, 6), (2, 3))   # slot ranges [s0, s1): the batch's counters carry on from call to call
    n0 = pool.stats()["fused_launches"]
    for s0, s1 in calls:
        pool.set_option("fused_max_tasks", 0)
        pool.delta(batch, s0, xd[s0:s1], v_two[s0:s1], y_two[s0:s1], case.stream)
        pool.set_option("fused_max_tasks", 1 << 20)
        pool.delta(batch, s0, xd[s0:s1], v_one[s0:s1], y_one[s0:s1], case.stream)
    pool.batch_end(batch)
    torch.cuda.synchronize()
    st = pool.stats()
    assert st["fused_launches"] - n0 == len(calls) and st["fused_timeouts"] == 0
    for s in range(lay.n_slots):
        assert torch.equal(v_one[s], v_two[s]), "slot %d: v differs between the one-launch and the two-launch form" % s
        assert torch.equal(y_one[s], y_two[s]), "slot %d: y differs between the one-launch and the two-launch form" % s
    # against the oracle: every slot was updated once per call that covered it
    for s in range(lay.n_slots):
        times = sum(1 for s0, s1 in calls if s0 <= s < s1)
        v_ref = case.opool.shrink(s, xs[s], t2a, acc64=True)
        y_ref = y0[s].copy()
        for _ in range(times):
            y_ref = case.opool.expand(s, v_ref, t2a, y_ref, acc64=True)
        err = rel_err(from_elt(torch_to_raw(y_one[s], lay.dtype), lay.dtype), from_elt(y_ref, lay.dtype))
        assert err <= times * TOL_Y[lay.dtype], "slot %d: y error %.3g after %d updates" % (s, err, times)
    case.close()


def test_a_wait_cut_short_from_the_host_ends_the_launch_and_is_counted(oracle_mod):
    import torch
    case, lay, ranks = _setup(oracle_mod)
    pool = case.gpool
    rng = np.random.default_rng(6)
    T = 300
    t2a = draw_tok2adapter(rng, T, np.arange(len(ranks)), s=1.0)
    xd = [raw_to_torch(make_act(rng, T, d, lay.dtype), "cuda") for d in lay.d_in]
    yd = [raw_to_torch(make_act(rng, T, d, lay.dtype), "cuda") for d in lay.d_out]
    vd = [torch.empty((T, case.max_rank), device="cuda") for _ in lay.d_in]
    pool.set_option("fused_max_tasks", 1 << 20)
    pool.set_option("fused_spin_limit", 0)          # one look at the flag, no waiting
    batch = pool.batch_begin(t2a, case.stream)
    print("launch with a single poll per expand task", flush=True)
    pool.delta(batch, 0, xd[:2], vd[:2], yd[:2], case.stream)
    torch.cuda.synchronize()                        # the launch ends although tasks found their slot unfinished
    st = pool.stats()
    print("given up:", st["fused_timeouts"], flush=True)
    assert st["fused_launches"] == 1 and st["fused_timeouts"] > 0
    pool.batch_end(batch)
    pool.set_option("fused_spin_limit", 1 << 20)
    out = case.run(t2a, seed=3)                     # the pool and the batch machinery are as good as before
    assert max(o["err_y"] for o in out) <= TOL_Y[lay.dtype]
    case.close()


def test_a_capturing_stream_takes_the_two_launches(oracle_mod):
    import torch
    case, lay, ranks = _setup(oracle_mod)
    pool = case.gpool
    pool.set_option("fused_max_tasks", 1 << 20)
    rng = np.random.default_rng(7)
    T = 64
    t2a = draw_tok2adapter(rng, T, np.arange(len(ranks)), s=1.0)
    xs = [make_act(rng, T, d, lay.dtype) for d in lay.d_in]
    y0 = [make_act(rng, T, d, lay.dtype) for d in lay.d_out]
    xd = [raw_to_torch(a, "cuda") for a in xs]
    y_init = [raw_to_torch(a, "cuda") for a in y0]
    yd = [t.clone() for t in y_init]
    vd = [torch.empty((T, case.max_rank), device="cuda") for _ in xs]
    side = torch.cuda.Stream()
    batch = pool.batch_begin(t2a, side.cuda_stream)
    pool.delta(batch, 0, xd, vd, yd, side.cuda_stream)        # eager: one launch
    torch.cuda.synchronize()
    y_eager = [t.clone() for t in yd]
    assert pool.stats()["fused_launches"] == 1
    for t, src in zip(yd, y_init):
        t.copy_(src)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        pool.delta(batch, 0, xd, vd, yd, side.cuda_stream)    # captured: shrink kernels, then expand kernels
    assert pool.stats()["fused_launches"] == 1
    for replay in range(3):
        for t, src in zip(yd, y_init):
            t.copy_(src)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for s in range(lay.n_slots):
            assert torch.equal(yd[s], y_eager[s]), "replay %d, slot %d" % (replay, s)
    pool.batch_end(batch)
    case.close()
