"""A step whose tensor table is already on the device is kernel launches only, so a caller can record it into
a HIP graph: recorded here through torch's stream capture, replayed several times with eager work and
synchronisations of the program in between, and every replay compared with the eager run of the same calls
(a recorded launch repeats the step number it was recorded with).  Both schedules: the ticket counter has to
reset itself between replays, since nothing outside the kernel touches it."""
import numpy as np
import pytest
import torch

import paper_2604_06836_amd as stq
from workloads import configs
from workloads.harness import DeviceModel, hparams

pytestmark = pytest.mark.gpu


def snapshot(dm):
    return [tuple(a.copy() for a in dm.host_state(l)) for l in range(len(dm.numel))]


def same(a, b, tag):
    for l, (x, y) in enumerate(zip(a, b)):
        for name, u, v in zip(("param", "m codes", "m scales", "v codes", "v scales"), x, y):
            assert np.array_equal(u.view(np.uint32), v.view(np.uint32)), f"{tag}: tensor {l} {name}"


@pytest.mark.parametrize("tickets,kind", [(False, "grad"), (True, "grad"), (True, True)])
def test_recorded_step_replays_like_the_eager_step(tickets, kind):
    w = configs.Workload(85, "graph", [("a", 30 * 2048 + 99), ("b", 4097), ("c", 12 * 2048)], 128, "bf16", 1,
                         "normal_per_tensor")
    plan = [(5, 4), (8, 3), (4, 6)]
    side = torch.cuda.Stream()
    ctxs = [stq.Context(0, 8), stq.Context(0, 8)]
    try:
        for c in ctxs:
            c.set_schedule(1 if tickets else 2 ** 63)
        with torch.cuda.stream(side):   # DeviceModel takes the current stream: everything on `side`
            ref, rec = DeviceModel(ctxs[0], w, plan), DeviceModel(ctxs[1], w, plan)
            for dm in (ref, rec):
                dm.set_grads(1)
                dm.step(1)              # uploads the tensor table on this stream
            side.synchronize()
            same(snapshot(ref), snapshot(rec), "before recording")
            hp = hparams(w, 2, kind)    # the recorded step also gathers statistics: the gradient's, or all
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                rec.ctx.step(rec.tensors, rec.cplan, hp, side.cuda_stream)
            for replay in range(4):
                graph.replay()
                ref.ctx.step(ref.tensors, ref.cplan, hp, side.cuda_stream)
                side.synchronize()
                same(snapshot(ref), snapshot(rec), f"replay {replay}")
                # eager work of the program between the replays
                junk = torch.ones(1 << 20, device="cuda")
                junk.mul_(2.0)
                side.synchronize()
            a, b = ref.ctx.stats(3, side.cuda_stream), rec.ctx.stats(3, side.cuda_stream)
            # (the recorded launches are not counted by the host: their statistics are read as one step's)
            for l in range(3):
                assert abs(a[l].g_sq_sum - b[l].g_sq_sum) <= 1e-12 * a[l].g_sq_sum and a[l].g_absmax == b[l].g_absmax
                assert abs(a[l].m_sq_sum - b[l].m_sq_sum) <= 1e-6 * a[l].m_sq_sum and a[l].v_absmax == b[l].v_absmax
                assert (a[l].m_sq_sum > 0) == (kind is True)
    finally:
        for c in ctxs:
            c.close()
