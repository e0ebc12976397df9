"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (all tensors of the workload in one stq_step call).

The last test does the same for the device-resident loop (stq_engine_step).

The oracle cannot run 10^9 elements in seconds, but blocks are independent: for sampled windows of
whole tiles (and every sampled tensor's ragged last tile) the inputs are copied to the host before
the step, the oracle is run on the window alone, and codes, scales and parameters of the window are
compared as in the small tests.  Gradient statistics of whole tensors are checked against float64
torch reductions on the device.
"""
import numpy as np
import pytest
import torch

import paper_2604_06836_amd as stq
from workloads import configs
from workloads.harness import DeviceModel

pytestmark = pytest.mark.gpu

TILE = 2048


def sample_windows(w, rng, n_tensors=10, per_tensor=3, tiles=2):
    """[(tensor index, first element, length)] : windows of whole tiles plus the ragged tails."""
    L = len(w.tensors)
    sizes = np.array([n for _, n in w.tensors])
    picks = {int(np.argmax(sizes)), int(np.argmin(sizes)), 0, L - 1}
    picks |= {int(i) for i in rng.choice(L, size=min(n_tensors, L), replace=False)}
    out = []
    for l in sorted(picks):
        n = int(sizes[l])
        nt = (n + TILE - 1) // TILE
        starts = {0, max(0, nt - tiles)} | {int(x) for x in rng.integers(0, nt, size=per_tensor)}
        for t0 in sorted(starts):
            lo = t0 * TILE
            out.append((l, lo, min(tiles * TILE, n - lo)))
    return out


def coverage_windows(w, rng, whole_below=1 << 20, frac=0.01, tiles=64, whole_budget=40_000_000):
    """Windows that cover every tensor of the workload: tensors below `whole_below` elements whole (up
    to `whole_budget` elements in all), of every other tensor its first and last `tiles` tiles (the ragged
    tail included) and random runs of `tiles` tiles until at least `frac` of the tensor is covered."""
    out, spent = [], 0
    for l, (_, n) in enumerate(w.tensors):
        nt = (n + TILE - 1) // TILE
        if n <= whole_below and spent + n <= whole_budget:
            out.append((l, 0, n))
            spent += n
            continue
        want = max(2, int(np.ceil(frac * nt / tiles)))
        starts = {0, max(0, nt - tiles)}
        while len(starts) < want:
            starts.add(int(rng.integers(0, max(1, nt - tiles))))
        merged_end = -1
        for t0 in sorted(starts):   # runs may not overlap: each window is compared on its own
            t0 = max(t0, merged_end)
            if t0 >= nt:
                continue
            lo = t0 * TILE
            out.append((l, lo, min(tiles * TILE, n - lo)))
            merged_end = t0 + tiles
    return out


def oracle_threads():
    import os
    return max(1, min(16, os.cpu_count() or 1))


def parallel(fn, items):
    """fn over items on the machine's cores (the oracle's C routines release the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=oracle_threads()) as ex:
        return list(ex.map(fn, items))


def window_state(oracle, dm, w, l, lo, n):
    """Host copy of one window of tensor l: params, grads and the unpacked oracle state."""
    bm, bv = dm.plan[l]
    K = w.K
    t0, nt = lo // TILE, (n + TILE - 1) // TILE
    th = dm.param[l][lo:lo + n].cpu().numpy().copy()
    g = dm.grad[l][lo:lo + n]
    g = g.view(torch.int16).cpu().numpy().view(np.uint16).copy() if g.dtype == torch.bfloat16 else g.cpu().numpy().copy()
    mw = dm.m_codes[l][t0 * 64 * bm:(t0 + nt) * 64 * bm].cpu().numpy().view(np.uint32)
    vw = dm.v_codes[l][t0 * 64 * bv:(t0 + nt) * 64 * bv].cpu().numpy().view(np.uint32)
    spt = TILE // K
    nb = (n + K - 1) // K
    ms = dm.m_scales[l][t0 * spt:t0 * spt + nb].cpu().numpy().copy()
    vs = dm.v_scales[l][t0 * spt:t0 * spt + nb].cpu().numpy().copy()
    st = oracle.State(n, K, bm, bv, um=oracle.unpack(mw, n, bm), sm=ms, cv=oracle.unpack(vw, n, bv), sv=vs)
    return th, g, st


def check_window(oracle, dm, w, l, lo, n, th_ref, st_ref, tag):
    bm, bv = dm.plan[l]
    t0, nt = lo // TILE, (n + TILE - 1) // TILE
    spt = TILE // w.K
    mw = dm.m_codes[l][t0 * 64 * bm:(t0 + nt) * 64 * bm].cpu().numpy().view(np.uint32)
    vw = dm.v_codes[l][t0 * 64 * bv:(t0 + nt) * 64 * bv].cpu().numpy().view(np.uint32)
    assert np.array_equal(mw, oracle.pack(st_ref.um, bm)), f"{tag}: m codes"
    assert np.array_equal(vw, oracle.pack(st_ref.cv, bv)), f"{tag}: v codes"
    ms = dm.m_scales[l][t0 * spt:(t0 + nt) * spt].cpu().numpy()
    vs = dm.v_scales[l][t0 * spt:(t0 + nt) * spt].cpu().numpy()
    assert np.array_equal(ms.view(np.uint32), oracle.pad_scales(st_ref.sm, n, w.K).view(np.uint32)), f"{tag}: m scales"
    assert np.array_equal(vs.view(np.uint32), oracle.pad_scales(st_ref.sv, n, w.K).view(np.uint32)), f"{tag}: v scales"
    th = dm.param[l][lo:lo + n].cpu().numpy()
    assert np.all(np.abs(th.astype(np.float64) - th_ref) <= 1e-6 * np.abs(th_ref)), f"{tag}: params"
    assert np.array_equal(th.view(np.uint32), th_ref.view(np.uint32)), f"{tag}: params not bit-equal"


def all_stats_close(g, o, tag):
    """Device statistics of a tensor against the oracle's: counts and maxima equal, the gradient's sums (fp64 on
    both sides) to 1e-12, the moments' sums (fp32 partial sums on the device) to 1e-5 plus the underflow floor."""
    assert g.count == o.count, tag
    for name in ("g_absmax", "m_absmax", "v_absmax"):
        assert getattr(g, name) == getattr(o, name), f"{tag} {name}"
    for name, scale in (("g_sum", o.g_abs_sum), ("g_abs_sum", o.g_abs_sum), ("g_sq_sum", o.g_sq_sum)):
        assert abs(getattr(g, name) - getattr(o, name)) <= 1e-12 * scale, f"{tag} {name}"
    for name, scale in (("m_sum", np.sqrt(o.m_sq_sum * o.count)), ("m_sq_sum", o.m_sq_sum), ("m_err_sq", o.m_err_sq),
                        ("v_sum", o.v_sum), ("v_sq_sum", o.v_sq_sum), ("v_err_sq", o.v_err_sq)):
        a, b = getattr(g, name), getattr(o, name)
        assert abs(a - b) <= 1e-5 * scale + o.count * 1.2e-38, f"{tag} {name}: {a} vs {b}"


@pytest.mark.parametrize("name", ["gpt2-small", "vit-b16", "gpt2-xl", "llama7b-slice"])
def test_full_size_sampled_parity(oracle, name):
    """Every tensor of the workload is covered: the small and medium ones whole, at least 1 % of each
    large one (first, last and random runs of 64 tiles); about 2-4 % of all elements per step."""
    w = configs.get_workload(name)
    rng = np.random.default_rng(1234 + w.cfg)
    plan = w.initial_plan()
    L = len(w.tensors)
    ctx = stq.Context(0, L)
    dm = DeviceModel(ctx, w, plan)
    windows = coverage_windows(w, rng)
    covered = sum(n for _, _, n in windows)
    assert covered >= 0.01 * w.numel and {l for l, _, _ in windows} == set(range(L))
    print(f"{name}: {len(windows)} windows, {covered} of {w.numel} elements per step", flush=True)
    for t in (1, 2, 3):
        dm.set_grads(t)
        want_stats = t == 3
        before = [window_state(oracle, dm, w, l, lo, n) for l, lo, n in windows]
        dm.step(t, stats=want_stats)
        torch.cuda.synchronize()
        ostats = parallel(lambda x: oracle.step(x[0], x[1], x[2], **w.hparams, t=t, want_stats=want_stats), before)
        for (l, lo, n), (th, g, st) in zip(windows, before):
            check_window(oracle, dm, w, l, lo, n, th, st, f"{name} step {t} tensor {l} window {lo}+{n}")
        print(f"{name}: step {t} compared", flush=True)
        if want_stats:
            gs = ctx.stats(L, dm.stream)
            for l in range(0, L, max(1, L // 24)):
                g64 = dm.grad[l].double()
                assert gs[l].count == g64.numel()
                assert abs(gs[l].g_sq_sum - float((g64 * g64).sum())) <= 1e-11 * float((g64 * g64).sum())
                assert abs(gs[l].g_abs_sum - float(g64.abs().sum())) <= 1e-11 * float(g64.abs().sum())
                assert abs(gs[l].g_sum - float(g64.sum())) <= 1e-11 * float(g64.abs().sum())
                assert gs[l].g_absmax == float(g64.abs().max())
                # the stored scales are the block maxima, so the maxima of the moments are the largest scales
                assert gs[l].m_absmax == float(dm.m_scales[l].max())
                assert gs[l].v_absmax == float(dm.v_scales[l].max())
                assert gs[l].m_err_sq <= gs[l].m_sq_sum and gs[l].v_err_sq <= gs[l].v_sq_sum
                del g64
            # the tensors that one window covers whole: all thirteen statistics against the oracle's
            whole = [(l, o) for (l, lo, n), o in zip(windows, ostats) if lo == 0 and n == w.tensors[l][1]]
            assert whole
            for l, o in whole:
                all_stats_close(gs[l], o, f"{name} tensor {l}")
            print(f"{name}: statistics of {len(whole)} whole tensors compared", flush=True)
    ctx.close()
    del dm
    torch.cuda.empty_cache()


def codes_window(buf, lo, n, b):
    t0, nt = lo // TILE, (n + TILE - 1) // TILE
    return buf[t0 * 64 * b:(t0 + nt) * 64 * b].cpu().numpy().view(np.uint32)


def test_repack_many_at_full_size(oracle):
    """stq_repack_many as the gpt2-xl configuration words its step (statistics, decision, re-pack of the
    changed states, then the step): all 388 tensors, a new plan that changes most states, so one launch of
    several hundred jobs and more than a million tiles (the kernel's grid-stride loop runs many times and
    its waves cross job boundaries).  Windows of every job -- whole small tensors, first, last and random
    runs of tiles of the large ones -- are compared with the oracle's re-pack of the same stored codes; then
    the step at the new widths is compared as in the test above."""
    w = configs.get_workload("gpt2-xl")
    rng = np.random.default_rng(777)
    L = len(w.tensors)
    plan = w.initial_plan()
    ctx = stq.Context(0, L)
    dm = DeviceModel(ctx, w, plan, spare_width=8)
    for t in (1, 2):   # two steps, so that the stored codes are not the initial pattern
        dm.set_grads(t)
        dm.step(t)
    torch.cuda.synchronize()
    # the new plan: every width moves to another member of the configuration's set, except for a few tensors
    widths = list(w.bits_m)
    new_plan = []
    for l, (bm, bv) in enumerate(plan):
        if l % 9 == 4:
            new_plan.append((bm, bv))
        else:
            new_plan.append((int(rng.choice([b for b in widths if b != bm])), int(rng.choice([b for b in widths if b != bv]))))
    windows = coverage_windows(w, rng, frac=0.005)
    jobs_expected = sum((a[0] != b[0]) + (a[1] != b[1]) for a, b in zip(plan, new_plan))
    tiles_expected = sum(((n + TILE - 1) // TILE) * ((a[0] != b[0]) + (a[1] != b[1]))
                         for (_, n), a, b in zip(w.tensors, plan, new_plan))
    assert jobs_expected > 600 and tiles_expected > 1_000_000
    old_codes = []
    for l, lo, n in windows:
        bm, bv = plan[l]
        old_codes.append((oracle.unpack(codes_window(dm.m_codes[l], lo, n, bm), n, bm),
                          oracle.unpack(codes_window(dm.v_codes[l], lo, n, bv), n, bv)))
    assert dm.apply_plan(new_plan) == jobs_expected
    torch.cuda.synchronize()
    print(f"re-packed {jobs_expected} states, {tiles_expected} tiles in one launch; {len(windows)} windows", flush=True)

    def expected(i):
        (l, lo, n), (um, cv) = windows[i], old_codes[i]
        (bm0, bv0), (bm1, bv1) = plan[l], new_plan[l]
        em = oracle.pack(oracle.repack(um, 0, bm0, bm1) if bm0 != bm1 else um, bm1)
        ev = oracle.pack(oracle.repack(cv, 1, bv0, bv1) if bv0 != bv1 else cv, bv1)
        return em, ev

    exp = parallel(expected, range(len(windows)))
    for (l, lo, n), (em, ev) in zip(windows, exp):
        bm1, bv1 = new_plan[l]
        assert np.array_equal(codes_window(dm.m_codes[l], lo, n, bm1), em), f"tensor {l} window {lo}+{n}: m codes {plan[l][0]}->{bm1}"
        assert np.array_equal(codes_window(dm.v_codes[l], lo, n, bv1), ev), f"tensor {l} window {lo}+{n}: v codes {plan[l][1]}->{bv1}"
    # the step that follows, at the new widths, on the re-packed states
    dm.set_grads(3)
    before = [window_state(oracle, dm, w, l, lo, n) for l, lo, n in windows]
    dm.step(3, stats=True)
    torch.cuda.synchronize()
    parallel(lambda x: oracle.step(x[0], x[1], x[2], **w.hparams, t=3), before)
    for (l, lo, n), (th, g, st) in zip(windows, before):
        check_window(oracle, dm, w, l, lo, n, th, st, f"after re-pack: tensor {l} window {lo}+{n}")
    ctx.close()
    del dm
    torch.cuda.empty_cache()


def test_switching_widths_every_five_steps_at_full_size(oracle):
    """The vit-b16 configuration as worded, at full size: 50 tensors, every 5 steps 10 % of them change one
    state's width through stq_repack_many (DeviceModel.apply_plan), then the step runs at the new widths.
    Eleven steps (switches before steps 5 and 10).  The oracle follows on windows that cover every tensor:
    its own re-pack at the switches, its own step every step; codes, scales and parameters are compared
    after every step."""
    w = configs.get_workload("vit-b16")
    rng = np.random.default_rng(4242)
    L = len(w.tensors)
    plan = w.initial_plan()
    ctx = stq.Context(0, L)
    dm = DeviceModel(ctx, w, plan, spare_width=8)
    windows = coverage_windows(w, rng, frac=0.01, tiles=32)
    ref = None
    switched = 0
    for t in range(1, 12):
        dm.set_grads(t)
        new_plan = w.switch_plan(plan, t)
        if ref is None:
            ref = [window_state(oracle, dm, w, l, lo, n) for l, lo, n in windows]
        else:   # the oracle keeps its own state from step to step; only the gradients come from the device
            for i, (l, lo, n) in enumerate(windows):
                ref[i] = (ref[i][0], dm.grad[l][lo:lo + n].cpu().numpy().copy(), ref[i][2])
        if new_plan != plan:
            switched += dm.apply_plan(new_plan)
            for (l, lo, n), (th, g, st) in zip(windows, ref):
                bm1, bv1 = new_plan[l]
                if bm1 != st.bm:
                    st.um, st.bm = oracle.repack(st.um, 0, st.bm, bm1), bm1
                if bv1 != st.bv:
                    st.cv, st.bv = oracle.repack(st.cv, 1, st.bv, bv1), bv1
            plan = new_plan
        dm.step(t)
        torch.cuda.synchronize()
        parallel(lambda x: oracle.step(x[0], x[1], x[2], **w.hparams, t=t), ref)
        for (l, lo, n), (th, g, st) in zip(windows, ref):
            check_window(oracle, dm, w, l, lo, n, th, st, f"vit-b16 step {t} tensor {l} window {lo}+{n}")
    assert switched >= 10
    ctx.close()
    del dm
    torch.cuda.empty_cache()


def test_tensor_beyond_2_31_elements(oracle):
    """One tensor of 2^31 + 4099 elements next to a small one: element, byte and code-word offsets
    pass 2^31 and 2^32.  Windows around those boundaries and the ragged tail are compared with the oracle."""
    n_big = (1 << 31) + 4099
    w = configs.Workload(97, "huge", [("small", 70_001), ("big", n_big)], 64, "bf16", 2, "normal")
    plan = [(5, 6), (8, 3)]
    ctx = stq.Context(0, 4)
    dm = DeviceModel(ctx, w, plan, init_params=False)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(12345)
    for l in range(2):
        dm.param[l].normal_(0.0, 0.02, generator=gen)
    nt = (n_big + TILE - 1) // TILE
    tiles = [0, (1 << 29) // TILE - 1, (1 << 30) // TILE - 1, (1 << 31) // TILE - 2, (1 << 31) // TILE - 1, nt - 2]
    windows = [(0, 0, 70_001)] + [(1, t0 * TILE, min(2 * TILE, n_big - t0 * TILE)) for t0 in tiles]
    for t in (1, 2):
        for l in range(2):   # gradients drawn on the device: the host generator would take minutes here
            dm.grad[l].copy_(torch.empty(dm.grad[l].numel(), dtype=torch.float32, device="cuda")
                             .normal_(0.0, 1e-3 * (l + 1), generator=gen))
        before = [window_state(oracle, dm, w, l, lo, n) for l, lo, n in windows]
        dm.step(t, stats=(t == 2))
        torch.cuda.synchronize()
        for (l, lo, n), (th, g, st) in zip(windows, before):
            oracle.step(th, g, st, **w.hparams, t=t)
            check_window(oracle, dm, w, l, lo, n, th, st, f"huge step {t} tensor {l} window {lo}+{n}")
    gs = ctx.stats(2, dm.stream)
    assert gs[1].count == n_big and gs[0].count == 70_001
    g64 = dm.grad[1].double()
    assert abs(gs[1].g_sq_sum - float((g64 * g64).sum())) <= 1e-11 * float((g64 * g64).sum())
    assert gs[1].g_absmax == float(g64.abs().max())
    del g64
    ctx.close()
    del dm
    torch.cuda.empty_cache()


def _window_of(oracle, w, codes_m, codes_v, dm, l, lo, n, bm, bv):
    """Host copy of a window's state from explicit code buffers at explicit widths (quantized widths only)."""
    K, t0, nt = w.K, lo // TILE, (n + TILE - 1) // TILE
    mw = codes_m[t0 * 64 * bm:(t0 + nt) * 64 * bm].cpu().numpy().view(np.uint32)
    vw = codes_v[t0 * 64 * bv:(t0 + nt) * 64 * bv].cpu().numpy().view(np.uint32)
    spt, nb = TILE // K, (n + K - 1) // K
    ms = dm.m_scales[l][t0 * spt:t0 * spt + nb].cpu().numpy().copy()
    vs = dm.v_scales[l][t0 * spt:t0 * spt + nb].cpu().numpy().copy()
    return mw, vw, ms, vs


@pytest.mark.parametrize("alg1", [False, True])
def test_device_resident_loop_at_full_size(oracle, alg1):
    """stq_engine_step on all 388 gpt2-xl tensors, as bench.py --transition engine launches it (alg1: in
    Algorithm 1's written order, the decision of step t applied in step t).  Per step: sampled windows go
    through the oracle's width-changing step at the widths the engine wrote, and the decision itself is
    redone by the oracle from float64 reductions of every tensor's gradient."""
    from paper_2604_06836_amd import binding
    w = configs.get_workload("gpt2-xl")
    rng = np.random.default_rng(99)
    L = len(w.tensors)
    plan = [(4, 4)] * L
    ctx = stq.Context(0, L)
    dm = DeviceModel(ctx, w, plan, spare_width=8)
    by_ptr = {}
    for l in range(L):
        for buf in (dm.m_codes[l], dm.v_codes[l], dm._spare[(l, 0)], dm._spare[(l, 1)]):
            by_ptr[buf.data_ptr()] = buf
    second = [(dm._spare[(l, 0)].data_ptr(), dm._spare[(l, 1)].data_ptr()) for l in range(L)]
    thr, bits = (2.0, 5.0, 7.5, 10.0, 13.0), (2, 3, 4, 5, 6, 8)
    kw = dict(alpha=0.3, tau=4.0, v_offset=-0.5, thr=thr, bits=bits)
    eng = ctx.engine(dm.tensors, second, dm.cplan, 8, w.K, alg1_order=alg1, stream=dm.stream, **kw)
    ema = oracle.Ema(0.0, 0.0, 0.0)
    windows = sample_windows(w, rng, n_tensors=8, per_tensor=2)
    changed = 0
    try:
        for t in (1, 2, 3):
            dm.set_grads(t)
            info = eng.read(dm.stream)
            before = []
            for l, lo, n in windows:
                bm, bv = info["stored"][l]
                cm, cv = (by_ptr[p] for p in info["current"][l])
                mw, vw, ms, vs = _window_of(oracle, w, cm, cv, dm, l, lo, n, bm, bv)
                th = dm.param[l][lo:lo + n].cpu().numpy().copy()
                g = dm.grad[l][lo:lo + n].view(torch.int16).cpu().numpy().view(np.uint16).copy()
                st = oracle.State(n, w.K, bm, bv, um=oracle.unpack(mw, n, bm), sm=ms, cv=oracle.unpack(vw, n, bv), sv=vs)
                before.append((th, g, st))
            eng.step(hparams_of(w, t), 1, None, dm.stream)
            after = eng.read(dm.stream)
            if not alg1:
                assert after["stored"] == info["next"], f"step {t}: the step wrote other widths than decided"
            else:
                assert after["next"] == after["stored"], f"step {t}: nothing may stay pending"
            for (l, lo, n), (th, g, st) in zip(windows, before):
                bm, bv = after["stored"][l]
                oracle.step_transition(th, g, st, bm, bv, **w.hparams, t=t)
                cm, cv = (by_ptr[p] for p in after["current"][l])
                mw, vw, ms, vs = _window_of(oracle, w, cm, cv, dm, l, lo, n, bm, bv)
                tag = f"engine step {t} tensor {l} window {lo}+{n}"
                assert np.array_equal(mw, oracle.pack(st.um, bm)), tag + ": m codes"
                assert np.array_equal(vw, oracle.pack(st.cv, bv)), tag + ": v codes"
                assert np.array_equal(ms.view(np.uint32), st.sm.view(np.uint32)), tag + ": m scales"
                assert np.array_equal(vs.view(np.uint32), st.sv.view(np.uint32)), tag + ": v scales"
                got = dm.param[l][lo:lo + n].cpu().numpy()
                assert np.array_equal(got.view(np.uint32), th.view(np.uint32)), tag + ": params"
            # the decision, from float64 reductions of every gradient
            stats = []
            for l in range(L):
                g64 = dm.grad[l].double()
                s = oracle.Stats()
                s.count, s.g_sum, s.g_abs_sum, s.g_sq_sum = g64.numel(), float(g64.sum()), float(g64.abs().sum()), float((g64 * g64).sum())
                stats.append(s)
            bm_o, bv_o, sc = oracle.decide(ema, stats, t, **kw)
            assert np.allclose(after["score"], sc, rtol=0, atol=1e-8), f"step {t} scores"
            assert np.allclose(after["ema"], (ema.n_ema, ema.r_ema, ema.v_ema), rtol=1e-10, atol=0), f"step {t} EMAs"
            for l in range(L):
                near = any(abs(sc[l] - x) < 1e-7 or abs(sc[l] - 0.5 - x) < 1e-7 for x in thr)
                if not near:   # by-product order: the widths the next step writes; written order: this step's
                    assert after["next"][l] == (int(bm_o[l]), int(bv_o[l])), f"step {t} tensor {l}: score {sc[l]}"
            changed += sum(a != b for a, b in zip(after["next"], info["stored"]))
        assert changed > L // 4   # widths really moved
    finally:
        eng.close()
        ctx.close()
    del dm
    torch.cuda.empty_cache()


def hparams_of(w, t):
    from workloads.harness import hparams
    return hparams(w, t)
