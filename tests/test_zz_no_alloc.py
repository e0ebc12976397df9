"""stq_step_static, the entry point that allocates nothing (its tensor table lives in a static device
array of the library), against stq_step on the same inputs: parameters, codes and scales must be bit-equal.
Two calls in a row on one context, the second with fewer and smaller tensors, so that the static table still
holds entries of the first call when the second one runs."""
import numpy as np
import pytest
import torch

import paper_2604_06836_amd as stq
from workloads import configs
from workloads.harness import DeviceModel, hparams

pytestmark = pytest.mark.gpu


def run(ctx, w, plan, steps, static, stats=False):
    dm = DeviceModel(ctx, w, plan)
    out = []
    for t in range(1, steps + 1):
        dm.set_grads(t)
        hp = hparams(w, t, stats)
        if static:
            ctx.step_static(dm.tensors, dm.cplan, hp, dm.stream)
        else:
            ctx.step(dm.tensors, dm.cplan, hp, dm.stream)
    torch.cuda.synchronize()
    for l in range(len(w.tensors)):
        out.append(dm.host_state(l))
    st = ctx.stats(len(w.tensors), dm.stream) if stats else None
    return out, st


def same(a, b, tag):
    for l, (x, y) in enumerate(zip(a, b)):
        for name, u, v in zip(("param", "m codes", "m scales", "v codes", "v scales"), x, y):
            assert np.array_equal(u.view(np.uint32), v.view(np.uint32)), f"{tag}: tensor {l} {name}"


def test_static_table_step_equals_step_twice_in_a_row():
    big = configs.Workload(81, "static-a", [("a", 40 * 2048 + 333), ("b", 5000), ("c", 1), ("d", 9 * 2048), ("e", 70_001)],
                           128, "bf16", 3, "normal_per_tensor")
    plan_big = [(8, 4), (5, 3), (2, 2), (6, 6), (4, 5)]
    small = configs.Workload(82, "static-b", [("a", 3 * 2048 + 17), ("b", 777)], 64, "fp32", 2, "normal_per_tensor")
    plan_small = [(3, 8), (7, 4)]
    ctx = stq.Context(0, 8)
    try:
        ref_big, ref_stats = run(ctx, big, plan_big, 3, static=False, stats=True)
        ref_small, _ = run(ctx, small, plan_small, 2, static=False)
        got_big, got_stats = run(ctx, big, plan_big, 3, static=True, stats=True)      # first call(s): 5 tensors
        got_small, _ = run(ctx, small, plan_small, 2, static=True)                    # then a smaller input
        same(ref_big, got_big, "5 tensors")
        same(ref_small, got_small, "2 tensors after 5")
        for l in range(len(big.tensors)):
            assert got_stats[l].count == ref_stats[l].count
            assert got_stats[l].g_absmax == ref_stats[l].g_absmax and got_stats[l].v_absmax == ref_stats[l].v_absmax
            assert abs(got_stats[l].g_sq_sum - ref_stats[l].g_sq_sum) <= 1e-9 * ref_stats[l].g_sq_sum
        # and once more the larger input, after the smaller one
        again, _ = run(ctx, big, plan_big, 3, static=True, stats=True)
        same(ref_big, again, "5 tensors after 2")
        # the ticket schedule of large launches, forced here: its scheduling words live in the static array too
        ctx.set_schedule(1)
        ref_t, ref_ts = run(ctx, big, plan_big, 3, static=False, stats="grad")
        got_t, got_ts = run(ctx, big, plan_big, 3, static=True, stats="grad")
        got_s, _ = run(ctx, small, plan_small, 2, static=True)
        same(ref_big, ref_t, "tickets against stripes")
        same(ref_t, got_t, "5 tensors, tickets")
        same(ref_small, got_s, "2 tensors after 5, tickets")
        for l in range(len(big.tensors)):
            assert got_ts[l].count == ref_ts[l].count and got_ts[l].g_absmax == ref_ts[l].g_absmax
            assert abs(got_ts[l].g_sq_sum - ref_ts[l].g_sq_sum) <= 1e-12 * ref_ts[l].g_sq_sum
    finally:
        ctx.close()


def test_static_table_limit_and_argument_checks():
    w = configs.Workload(83, "static-c", [("a", 100)], 128, "fp32", 1, "normal")
    ctx = stq.Context(0, 2048)
    try:
        dm = DeviceModel(ctx, w, [(4, 4)])
        n = 1025  # one more than STQ_STATIC_MAX_TENSORS
        many = (type(dm.tensors[0]) * n)(*([dm.tensors[0]] * n))
        plan = (type(dm.cplan[0]) * n)(*([dm.cplan[0]] * n))
        with pytest.raises(stq.StqError) as e:
            ctx.step_static(many, plan, hparams(w, 1), dm.stream)
        assert e.value.code == -8 and "static" in str(e.value)
        hp = hparams(w, 1)
        hp.block = 100
        with pytest.raises(stq.StqError) as e:
            ctx.step_static(dm.tensors, dm.cplan, hp, dm.stream)
        assert e.value.code == -4
        torch.cuda.synchronize()
    finally:
        ctx.close()
