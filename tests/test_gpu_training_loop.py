"""End-to-end use of the library as an optimizer: a small regression model trained with the
quantized Adam step, the statistics -> decision -> width-change loop of Algorithm 1 running at its
update cadence, compared with torch's fp32 AdamW on the same data and initial weights.

Two ladders: the paper's own {4, 8, 16, 32} starting from its initial width 16, and the same clamped
to the block-quantized widths (16 and 32 -> 8).  The statistics of step t come out of step t's kernel, so a new plan takes effect at step t+1.
A second test runs the same loop through the device-resident engine (stq_engine_*).
No oracle here: this checks that the pieces work together as an optimizer (loss parity), the
element-wise parity of every piece is in the other GPU tests.
"""
import numpy as np
import pytest
import torch

import paper_2604_06836_amd as stq
from paper_2604_06836_amd import binding

pytestmark = pytest.mark.gpu

LR, BETAS, EPS, WD, K, U = 2e-3, (0.9, 0.999), 1e-8, 0.01, 128, 10


def make_model(seed):
    torch.manual_seed(seed)
    m = torch.nn.Sequential(torch.nn.Linear(32, 256), torch.nn.GELU(), torch.nn.Linear(256, 256), torch.nn.GELU(),
                            torch.nn.Linear(256, 1)).cuda()
    return m


def batches(steps, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    w = torch.randn(32, 3, device="cuda", generator=g) / 32 ** 0.5
    for _ in range(steps):
        x = torch.randn(512, 32, device="cuda", generator=g)
        h = x @ w
        y = torch.sin(h[:, :1]) + 0.5 * h[:, 1:2] * h[:, 2:3] + 0.05 * torch.randn(512, 1, device="cuda", generator=g)
        yield x, y


def train_fp32(steps):
    m = make_model(0)
    opt = torch.optim.AdamW(m.parameters(), lr=LR, betas=BETAS, eps=EPS, weight_decay=WD)
    losses = []
    for x, y in batches(steps, 1):
        opt.zero_grad(set_to_none=True)
        loss = torch.nn.functional.mse_loss(m(x), y)
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    return losses


def train_quantized(steps, fixed_plan=None, ladder=(4, 8, 8, 8), start=(8, 8)):
    m = make_model(0)
    params = [p for p in m.parameters()]
    L = len(params)
    ctx = stq.Context(0, L)
    stream = torch.cuda.current_stream().cuda_stream
    plan = [fixed_plan or start] * L
    bufs = []
    for p, (bm, bv) in zip(params, plan):
        n = p.numel()
        cm, sb = stq.state_bytes(n, K, max(ladder))   # code buffers sized for the widest width, two of each
        bufs.append(dict(m=[torch.empty(cm // 4, dtype=torch.int32, device="cuda") for _ in range(2)],
                         v=[torch.empty(cm // 4, dtype=torch.int32, device="cuda") for _ in range(2)],
                         ms=torch.empty(sb // 4, dtype=torch.float32, device="cuda"),
                         vs=torch.empty(sb // 4, dtype=torch.float32, device="cuda"), cur=[0, 0]))

    def tensors():
        return binding.make_tensors(dict(param=p.data_ptr(), grad=(p.grad.data_ptr() if p.grad is not None else None),
                                         numel=p.numel(), m_codes=b["m"][b["cur"][0]].data_ptr(), m_scales=b["ms"].data_ptr(),
                                         v_codes=b["v"][b["cur"][1]].data_ptr(), v_scales=b["vs"].data_ptr())
                                    for p, b in zip(params, bufs))

    ctx.zero_state(tensors(), binding.make_plan(plan), K, stream)
    ema = binding.DecideState(0, 0, 0)
    pending, losses, widths = None, [], []
    for t, (x, y) in enumerate(batches(steps, 1), start=1):
        for p in params:
            p.grad = None
        loss = torch.nn.functional.mse_loss(m(x), y)
        loss.backward()
        losses.append(float(loss.detach()))
        due = fixed_plan is None and binding.decide_due(t, U)
        hp = binding.HParams(LR, BETAS[0], BETAS[1], EPS, WD, t, K, 0, stq.STQ_FLAG_STATS if due else 0)
        if pending is not None and pending != plan:
            dests = []
            for b, (bm0, bv0), (bm1, bv1) in zip(bufs, plan, pending):
                dm = b["m"][1 - b["cur"][0]].data_ptr() if bm0 != bm1 else None
                dv = b["v"][1 - b["cur"][1]].data_ptr() if bv0 != bv1 else None
                dests.append((dm, dv))
            ctx.step_transition(tensors(), binding.make_plan(plan), binding.make_plan(pending), dests, hp, stream)
            for b, (bm0, bv0), (bm1, bv1) in zip(bufs, plan, pending):
                if bm0 != bm1:
                    b["cur"][0] ^= 1
                if bv0 != bv1:
                    b["cur"][1] ^= 1
            plan = pending
        else:
            ctx.step(tensors(), binding.make_plan(plan), hp, stream)
        pending = None
        if due:
            st = ctx.stats(L, stream)
            new_plan, _ = stq.decide(ema, st, t, alpha=0.1, tau=100.0, thr=(6.8, 12.0, 24.0), bits=ladder)
            pending = [tuple(int(b) for b in p) for p in new_plan]
        widths.append(np.mean([bm + bv for bm, bv in plan]) / 2)
    torch.cuda.synchronize()
    ctx.close()
    return losses, widths


def train_engine(steps, ladder=(4, 8, 16, 32), start=(16, 16), alg1=False):
    """The same loop through stq_engine_*: the host enqueues one call per step and never reads anything back."""
    m = make_model(0)
    params = [p for p in m.parameters()]
    L = len(params)
    ctx = stq.Context(0, L)
    stream = torch.cuda.current_stream().cuda_stream
    cap = max(max(ladder), *start)
    keep = []
    for p in params:
        cm, sb = stq.state_bytes(p.numel(), K, cap)
        keep.append(([torch.empty(cm // 4, dtype=torch.int32, device="cuda") for _ in range(4)],
                     [torch.empty(sb // 4, dtype=torch.float32, device="cuda") for _ in range(2)]))
    loss = torch.nn.functional.mse_loss(m(torch.zeros(1, 32, device="cuda")), torch.zeros(1, 1, device="cuda"))
    loss.backward()   # gradient buffers to create the engine with; each step passes its own
    tensors = binding.make_tensors(dict(param=p.data_ptr(), grad=p.grad.data_ptr(), numel=p.numel(),
                                        m_codes=c[0].data_ptr(), m_scales=s[0].data_ptr(),
                                        v_codes=c[1].data_ptr(), v_scales=s[1].data_ptr())
                                   for p, (c, s) in zip(params, keep))
    plan = binding.make_plan([start] * L)
    ctx.zero_state(tensors, plan, K, stream)
    eng = ctx.engine(tensors, [(c[2].data_ptr(), c[3].data_ptr()) for c, _ in keep], plan, cap, K,
                     alpha=0.1, tau=100.0, thr=(6.8, 12.0, 24.0), bits=ladder, alg1_order=alg1, stream=stream)
    losses = []
    for t, (x, y) in enumerate(batches(steps, 1), start=1):
        for p in params:
            p.grad = None
        loss = torch.nn.functional.mse_loss(m(x), y)
        loss.backward()
        losses.append(loss.detach())
        eng.step(binding.HParams(LR, BETAS[0], BETAS[1], EPS, WD, t, K, 0, 0), U, [p.grad.data_ptr() for p in params], stream)
    final = eng.read(stream)["stored"]
    eng.close()
    ctx.close()
    return [float(x) for x in losses], final


@pytest.mark.parametrize("alg1", [False, True])
def test_device_resident_loop_trains_like_fp32_adamw(alg1):
    # alg1: the decision of step t applied in step t (Algorithm 1's written order) instead of step t+1
    steps = 400
    ref = train_fp32(steps)
    host, _ = train_quantized(steps, ladder=(4, 8, 16, 32), start=(16, 16))
    dev, final = train_engine(steps, alg1=alg1)
    tail = lambda xs: float(np.mean(xs[-50:]))
    assert tail(dev) <= 1.25 * tail(ref) + 1e-3, (tail(dev), tail(ref))
    assert abs(tail(dev) - tail(host)) <= 0.05 * tail(host), (tail(dev), tail(host))   # same decisions, same path
    assert any(w != 16 for p in final for w in p) and all(w in (4, 8, 16, 32) for p in final for w in p)
    print("final losses: fp32 %.4f, host loop %.4f, device loop %.4f; final plan %s" % (tail(ref), tail(host), tail(dev), final))


def test_quantized_adam_trains_like_fp32_adamw():
    steps = 400
    ref = train_fp32(steps)
    q8, _ = train_quantized(steps, fixed_plan=(8, 8))
    dyn, widths = train_quantized(steps)
    paper, pw = train_quantized(steps, ladder=(4, 8, 16, 32), start=(16, 16))   # Algorithm 1's ladder and initial width
    tail = lambda xs: float(np.mean(xs[-50:]))
    assert tail(ref) < 0.35 * float(np.mean(ref[:10]))          # the reference run did learn
    assert tail(q8) <= 1.10 * tail(ref) + 1e-3, (tail(q8), tail(ref))
    assert tail(dyn) <= 1.25 * tail(ref) + 1e-3, (tail(dyn), tail(ref))   # widths fall to 4 bits on this toy problem
    assert tail(paper) <= 1.25 * tail(ref) + 1e-3, (tail(paper), tail(ref))
    assert min(widths) >= 4 and max(widths) <= 8
    assert len(set(widths)) > 1 and len(set(pw)) > 1             # the plans did change during training
    assert pw[0] == 16 and min(pw) >= 4 and max(pw) <= 32
    print("final losses: fp32 %.4f, 8-bit %.4f, dynamic %.4f, paper ladder %.4f; mean width %.2f .. %.2f, paper ladder %.2f .. %.2f"
          % (tail(ref), tail(q8), tail(dyn), tail(paper), min(widths), max(widths), min(pw), max(pw)))
