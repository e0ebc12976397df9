"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same seeded inputs.

Bar: packed codes and block scales bit-exact; parameters within 1e-6 relative (they are in fact
produced by the same correctly rounded fp32 operations, so equality is also asserted where it
must hold).  Statistics: the gradient's sums (fp64 throughout) 1e-12 relative, the moments' sums (fp32 lane sums) 1e-5; maxima exact.
"""
import numpy as np
import pytest
import torch

import paper_2604_06836_amd as stq
from paper_2604_06836_amd import binding
from workloads import configs
from workloads.harness import DeviceModel, hparams

pytestmark = pytest.mark.gpu

PARAM_RTOL = 1e-6


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = stq.Context(0, 1024)
    yield c
    c.close()


def oracle_states(oracle, w, plan):
    return [oracle.State.zeros(n, w.K, bm, bv) for (_, n), (bm, bv) in zip(w.tensors, plan)]


def assert_tensor_parity(oracle, dm, l, th_ref, st_ref, tag=""):
    th, mw, ms, vw, vs = dm.host_state(l)
    n, K = st_ref.numel, st_ref.K
    want_m = oracle.pack_wide(st_ref.mw, st_ref.bm) if st_ref.bm >= 16 else oracle.pack(st_ref.um, st_ref.bm)
    want_v = oracle.pack_wide(st_ref.vw, st_ref.bv) if st_ref.bv >= 16 else oracle.pack(st_ref.cv, st_ref.bv)
    assert np.array_equal(mw, want_m), f"{tag} m codes tensor {l}"
    assert np.array_equal(vw, want_v), f"{tag} v codes tensor {l}"
    assert np.array_equal(ms.view(np.uint32), oracle.pad_scales(st_ref.sm, n, K).view(np.uint32)), f"{tag} m scales {l}"
    assert np.array_equal(vs.view(np.uint32), oracle.pad_scales(st_ref.sv, n, K).view(np.uint32)), f"{tag} v scales {l}"
    err = np.abs(th.astype(np.float64) - th_ref)
    assert np.all(err <= PARAM_RTOL * np.abs(th_ref)), f"{tag} params tensor {l}: max rel {np.max(err / np.maximum(np.abs(th_ref), 1e-30))}"
    # stronger than the bar: the kernel's square root and quotient are correctly rounded like the
    # oracle's, so the parameters agree bit for bit
    assert np.array_equal(th.view(np.uint32), th_ref.view(np.uint32)), f"{tag} params tensor {l}: {np.count_nonzero(th != th_ref)} not bit-equal"


def run_both(oracle, ctx, w, plan, steps, stats_steps=(), tag=""):
    dm = DeviceModel(ctx, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    for l in range(len(w.tensors)):  # initial state
        assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], tag + " init")
    for t in range(1, steps + 1):
        dm.set_grads(t)
        want_stats = t in stats_steps
        dm.step(t, stats=want_stats)
        torch.cuda.synchronize()
        gpu_stats = dm.ctx.stats(len(w.tensors), dm.stream) if want_stats else None
        for l in range(len(w.tensors)):
            s = oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t, want_stats=want_stats)
            assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"{tag} step {t}")
            if want_stats:
                assert_stats_close(gpu_stats[l], s, f"{tag} step {t} tensor {l}")
    return dm, th_ref, st_ref


def assert_stats_close(g, o, tag):
    assert g.count == o.count, tag
    for name in ("g_sum", "g_abs_sum", "g_sq_sum", "m_sum", "m_sq_sum", "m_err_sq", "v_sum", "v_sq_sum", "v_err_sq"):
        a, b = getattr(g, name), getattr(o, name)
        # signed sums cancel: compare against the scale of the absolute sum
        scale = {"g_sum": o.g_abs_sum, "m_sum": np.sqrt(o.m_sq_sum * o.count)}.get(name, abs(b))
        if name.startswith("g_"):
            # the gradient's sums are taken in fp64 from the first addition: only the order differs
            assert abs(a - b) <= 1e-12 * scale, f"{tag} {name}: {a} vs {b}"
            continue
        # the kernel adds the moments' terms in fp32 (a lane's 8 elements of a quarter, then eight lanes, then
        # the quarters of up to 16 tiles) before widening to fp64, so terms below the smallest normal fp32
        # (2^-126) lose bits: absolute floor of count * 2^-126
        assert abs(a - b) <= 1e-5 * scale + o.count * 1.2e-38, f"{tag} {name}: {a} vs {b}"
    for name in ("g_absmax", "m_absmax", "v_absmax"):
        assert getattr(g, name) == getattr(o, name), f"{tag} {name}"


# ------------------------------------------------------------------ configuration 1
def test_config1_full_size_all_steps(oracle, ctx):
    # 768x3072 fp32 tensor, m at 8 bits, v at 4 bits, K = 128, 10 steps: every element compared
    w = configs.get_workload("adam-1tensor")
    run_both(oracle, ctx, w, w.initial_plan(), w.steps, stats_steps=(1, 10), tag="cfg1")


# ------------------------------------------------- every width pair, every block size
@pytest.mark.parametrize("K", [64, 128, 256])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_all_width_pairs(oracle, ctx, K, dtype):
    # 49 tensors, one per (bm, bv), sizes spanning several tiles with ragged tails
    pairs = [(bm, bv) for bm in range(2, 9) for bv in range(2, 9)]
    rng = np.random.default_rng(K)
    sizes = [int(rng.integers(1, 4)) * 2048 + int(rng.integers(0, 2048)) for _ in pairs]
    w = configs.Workload(90, f"pairs-{K}-{dtype}", [(f"t{i}", n) for i, n in enumerate(sizes)], K, dtype, 3,
                         "normal_per_tensor")
    run_both(oracle, ctx, w, pairs, 3, stats_steps=(2,), tag=w.name)


# ------------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("numel", [1, 3, 63, 64, 65, 2047, 2048, 2049, 4096 + 129, 10 * 2048 + 1])
def test_ragged_sizes(oracle, ctx, numel):
    for K in (64, 256):
        w = configs.Workload(91, f"ragged-{numel}", [("a", numel), ("b", numel)], K, "fp32", 2, "normal")
        run_both(oracle, ctx, w, [(5, 3), (8, 2)], 2, stats_steps=(1, 2), tag=w.name)


def test_degenerate_values(oracle, ctx):
    # zero gradients, one huge outlier, denormal-sized gradients, a block of equal values
    n, K = 3 * 2048 + 700, 128
    w = configs.Workload(92, "degenerate", [("zero", n), ("outlier", n), ("tiny", n), ("equal", n)], K, "fp32", 3, "normal")
    plan = [(8, 4), (4, 4), (6, 5), (3, 8)]
    dm = DeviceModel(ctx, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    for t in range(1, 4):
        dm.set_grads(t)
        dm.grad[0].zero_()
        dm.grad[1][1000] = 3.0e4
        dm.grad[1][n - 1] = -7.0e3
        dm.grad[2].mul_(1e-17)          # g^2 ~ 1e-40: second moments below the smallest normal
        dm.grad[3].fill_(2.5e-4)
        dm.step(t, stats=True)
        torch.cuda.synchronize()
        gs = dm.ctx.stats(4, dm.stream)
        for l in range(4):
            s = oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t, want_stats=True)
            assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"degenerate step {t}")
            assert_stats_close(gs[l], s, f"degenerate step {t} tensor {l}")
    assert np.all(st_ref[0].sm == 0) and np.all(st_ref[0].sv == 0)  # the all-zero case really was all-zero
    assert np.all(st_ref[2].sv == 0)                                   # tiny blocks were flushed


def test_weight_decay_and_other_hparams(oracle, ctx):
    w = configs.Workload(93, "hp", [("a", 5000), ("b", 9000)], 128, "bf16", 4, "student_t")
    w.hparams = dict(lr=3e-4, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)
    run_both(oracle, ctx, w, [(6, 4), (4, 6)], 4, tag="hp")


# -------------------------------------------------------------------------- re-pack
@pytest.mark.parametrize("state", [0, 1])
def test_repack_every_width_pair(oracle, ctx, state):
    n = 2 * 2048 + 1234
    rng = np.random.default_rng(5 + state)
    for b_old in range(2, 9):
        hi = 2 ** b_old - (1 if state == 0 else 0)   # linear codes never use the top value
        codes = rng.integers(0, hi, n, dtype=np.uint8)
        src = torch.from_numpy(oracle.pack(codes, b_old).view(np.int32)).cuda()
        for b_new in range(2, 9):
            cb, _ = stq.state_bytes(n, 128, b_new)
            dst = torch.full((cb // 4,), -1, dtype=torch.int32, device="cuda")
            ctx.repack(n, 128, state, src.data_ptr(), b_old, dst.data_ptr(), b_new,
                       torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            want = oracle.pack(oracle.repack(codes, state, b_old, b_new), b_new)
            assert np.array_equal(dst.cpu().numpy().view(np.uint32), want), (state, b_old, b_new)


def test_repack_many_matches_oracle(oracle, ctx):
    # 40 width changes of both states in one launch: sizes from 1 element to several tiles, ragged
    # tails, every old/new width; destinations pre-filled so that unwritten words would show
    rng = np.random.default_rng(77)
    sizes = [1, 63, 2047, 2048, 2049, 5 * 2048 + 700, 12 * 2048, 3 * 2048 + 1]
    jobs, keep = [], []
    for i in range(40):
        n = sizes[i % len(sizes)] + (i // len(sizes)) * 17
        state = i % 2
        b_old = int(rng.integers(2, 9))
        b_new = int(rng.choice([b for b in range(2, 9) if b != b_old]))
        hi = 2 ** b_old - (1 if state == 0 else 0)
        codes = rng.integers(0, hi, n, dtype=np.uint8)
        src = torch.from_numpy(oracle.pack(codes, b_old).view(np.int32)).cuda()
        cb, _ = stq.state_bytes(n, 128, b_new)
        dst = torch.full((cb // 4,), -1, dtype=torch.int32, device="cuda")
        jobs.append((n, state, src.data_ptr(), b_old, dst.data_ptr(), b_new))
        keep.append((codes, src, dst, state, b_old, b_new))
    ctx.repack_many(jobs, 128, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for i, (codes, src, dst, state, b_old, b_new) in enumerate(keep):
        want = oracle.pack(oracle.repack(codes, state, b_old, b_new), b_new)
        assert np.array_equal(dst.cpu().numpy().view(np.uint32), want), (i, state, b_old, b_new)
    # rejected arguments
    lib = stq.load_library()
    n, state, src, b0, dst, b1 = jobs[5]
    def call(j, count=1):
        arr = (binding.RepackJob * 1)(binding.RepackJob(j[0], j[2], j[4], j[1], j[3], j[5]))
        return lib.stq_repack_many(ctx._h, arr, count, 128, None)
    assert call((n, state, src, 9, dst, b1)) == -3
    assert call((n, state, src, b0, dst + 4, b1)) == -2
    assert call((n, state, src, b0, src, b1)) == -1      # overlapping source and destination
    assert call((0, state, src, b0, dst, b1)) == -1
    assert call((n, 2, src, b0, dst, b1)) == -1
    assert call((n, state, src, b0, dst, b1), count=0) == -1


def test_transitions_config3_scaled(oracle, ctx):
    # ViT-shaped tensors (reduced), Student-t gradients, K = 256, widths switching every 5 steps
    w = configs.scaled(configs.get_workload("vit-b16"), 40_000, 12)
    plan = w.initial_plan()
    dm = DeviceModel(ctx, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    n_changed = 0
    for t in range(1, 13):
        new_plan = w.switch_plan(plan, t)
        if new_plan != plan:
            n_changed += dm.apply_plan(new_plan)
            for l, ((bm0, bv0), (bm1, bv1)) in enumerate(zip(plan, new_plan)):
                if bm0 != bm1:
                    st_ref[l].um = oracle.repack(st_ref[l].um, 0, bm0, bm1)
                    st_ref[l].bm = bm1
                if bv0 != bv1:
                    st_ref[l].cv = oracle.repack(st_ref[l].cv, 1, bv0, bv1)
                    st_ref[l].bv = bv1
            plan = new_plan
        dm.set_grads(t)
        dm.step(t)
        torch.cuda.synchronize()
        for l in range(len(w.tensors)):
            oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t)
            assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"cfg3 step {t}")
    assert n_changed >= 2


def test_decide_loop_config4_scaled(oracle, ctx):
    # GPT-2-XL-shaped tensors (reduced; d = 1600 keeps the ragged blocks), bf16 gradients; every step:
    # statistics -> decision -> re-pack -> step.  Both sides are driven by the ORACLE's plan; the plan
    # from the GPU statistics must agree wherever the score is not within 1e-4 of a threshold.
    w = configs.scaled(configs.get_workload("gpt2-xl"), 30_000, 14)
    L = len(w.tensors)
    ladder = dict(thr=(9.0, 11.0, 13.0, 15.0, 17.0), bits=(2, 3, 4, 5, 6, 8))
    plan = [(4, 4)] * L
    dm = DeviceModel(ctx, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    e_gpu, e_or = binding.DecideState(0, 0, 0), oracle.Ema(0, 0, 0)
    widths_seen = set()
    for t in range(1, 9):
        dm.set_grads(t)
        dm.step(t, stats=True)
        torch.cuda.synchronize()
        gs = dm.ctx.stats(L, dm.stream)
        os_ = []
        for l in range(L):
            os_.append(oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t, want_stats=True))
            assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"cfg4 step {t}")
            assert_stats_close(gs[l], os_[l], f"cfg4 step {t} tensor {l}")
        p_gpu, sc_gpu = stq.decide(e_gpu, gs, t, alpha=0.3, tau=4.0, v_offset=-1.0, **ladder)
        bm, bv, sc = oracle.decide(e_or, os_, t, alpha=0.3, tau=4.0, v_offset=-1.0, **ladder)
        new_plan = [(int(a), int(b)) for a, b in zip(bm, bv)]
        thr = np.array(ladder["thr"])
        for l in range(L):
            if min(np.min(np.abs(thr - sc[l])), np.min(np.abs(thr - (sc[l] - 1.0)))) > 1e-4:
                assert p_gpu[l] == new_plan[l]
        widths_seen |= {b for p in new_plan for b in p}
        dm.apply_plan(new_plan)
        for l, ((bm0, bv0), (bm1, bv1)) in enumerate(zip(plan, new_plan)):
            if bm0 != bm1:
                st_ref[l].um, st_ref[l].bm = oracle.repack(st_ref[l].um, 0, bm0, bm1), bm1
            if bv0 != bv1:
                st_ref[l].cv, st_ref[l].bv = oracle.repack(st_ref[l].cv, 1, bv0, bv1), bv1
        plan = new_plan
    assert len(widths_seen) >= 3


# ------------------------------------------------- scaled copies of configs 2 and 5
@pytest.mark.parametrize("name", ["gpt2-small", "llama7b-slice"])
def test_scaled_configs(oracle, ctx, name):
    w = configs.scaled(configs.get_workload(name), 50_000, 24)
    run_both(oracle, ctx, w, w.initial_plan(), 4, stats_steps=(4,), tag=name)


# ------------------------------------------------------- step with a change of widths
@pytest.mark.parametrize("dtype,K", [("fp32", 128), ("bf16", 64), ("fp32", 256)])
def test_step_transition_every_width_pair(oracle, ctx, dtype, K):
    # 49 tensors: tensor i changes m from 2+i//7 to 2+i%7 bits and v from 2+i%7 to 2+i//7 bits
    # (the diagonal keeps its widths and stays in place), after two ordinary steps; ragged sizes
    sizes = [3 * 2048 + 517, 2048, 4096 + 1, 700, 5 * 2048]
    tensors = [(f"t{i}", sizes[i % len(sizes)] + i) for i in range(49)]
    w = configs.Workload(95, f"trans-{dtype}-{K}", tensors, K, dtype, 4, "normal_per_tensor")
    old = [(2 + i // 7, 2 + i % 7) for i in range(49)]
    new = [(2 + i % 7, 2 + i // 7) for i in range(49)]
    dm = DeviceModel(ctx, w, old)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, old)
    for t in (1, 2):
        dm.set_grads(t)
        dm.step(t)
        for l in range(49):
            oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t)
    dm.set_grads(3)
    changed = dm.step_transition(3, new, stats=True)
    torch.cuda.synchronize()
    assert changed == 2 * 42
    gs = dm.ctx.stats(49, dm.stream)
    for l in range(49):
        s = oracle.step_transition(th_ref[l], dm.host_grad(l), st_ref[l], *new[l], **w.hparams, t=3, want_stats=True)
        assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"transition tensor {l} {old[l]}->{new[l]}")
        assert_stats_close(gs[l], s, f"transition tensor {l}")
    # and the model keeps stepping at the new widths
    dm.set_grads(4)
    dm.step(4)
    torch.cuda.synchronize()
    for l in range(49):
        oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=4)
        assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"after transition tensor {l}")


def test_step_transition_argument_checks(ctx):
    w = configs.Workload(96, "targs", [("a", 4096)], 128, "fp32", 1, "normal")
    dm = DeviceModel(ctx, w, [(8, 4)])
    lib = stq.load_library()
    import ctypes as C
    hp = hparams(w, 1)
    cb, _ = stq.state_bytes(4096, 128, 5)
    dst = torch.empty(cb // 4 + 64, dtype=torch.int32, device="cuda")

    def call(new_plan, m, v):
        arr = (binding.Codes * 1)(binding.Codes(m, v))
        return lib.stq_step_transition(ctx._h, dm.tensors, 1, dm.cplan, binding.make_plan(new_plan), arr, C.byref(hp), None)

    assert call([(5, 4)], None, None) == -1                           # a changed width needs a destination
    assert call([(5, 4)], dm.m_codes[0].data_ptr(), None) == -1      # ... that is not the source
    assert call([(5, 4)], dst.data_ptr() + 4, None) == -2            # ... and is aligned
    assert call([(9, 4)], dst.data_ptr(), None) == -3
    assert lib.stq_step_transition(ctx._h, dm.tensors, 1, dm.cplan, None, None, C.byref(hp), None) == -1
    assert call([(5, 4)], dst.data_ptr(), None) == 0
    torch.cuda.synchronize()


# ------------------------------------------------- the 16- and 32-bit members of the width set
WIDTHS = (4, 8, 16, 32)   # the paper's set B


@pytest.mark.parametrize("dtype,K", [("fp32", 128), ("bf16", 64)])
def test_wide_states_every_combination(oracle, ctx, dtype, K):
    # 16 tensors, one per (m width, v width) over {4, 8, 16, 32}; ragged sizes; statistics on
    sizes = [2 * 2048 + 333, 2048, 4096 + 1, 900]
    tensors = [(f"t{i}", sizes[i % 4] + 3 * i) for i in range(16)]
    plan = [(WIDTHS[i // 4], WIDTHS[i % 4]) for i in range(16)]
    w = configs.Workload(98, f"wide-{dtype}-{K}", tensors, K, dtype, 3, "normal_per_tensor")
    run_both(oracle, ctx, w, plan, 3, stats_steps=(1, 3), tag=w.name)


@pytest.mark.parametrize("dtype,K", [("fp32", 256), ("bf16", 128)])
def test_transitions_among_the_papers_widths(oracle, ctx, dtype, K):
    # tensor i: first moment WIDTHS[i//4] -> WIDTHS[i%4], second moment WIDTHS[i%4] -> WIDTHS[i//4]
    sizes = [3 * 2048 + 77, 2048, 4096 + 1, 650]
    tensors = [(f"t{i}", sizes[i % 4] + 5 * i) for i in range(16)]
    old = [(WIDTHS[i // 4], WIDTHS[i % 4]) for i in range(16)]
    new = [(WIDTHS[i % 4], WIDTHS[i // 4]) for i in range(16)]
    w = configs.Workload(99, f"wtrans-{dtype}-{K}", tensors, K, dtype, 4, "normal_per_tensor")
    dm = DeviceModel(ctx, w, old)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, old)
    for t in (1, 2):
        dm.set_grads(t)
        dm.step(t)
        for l in range(16):
            oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t)
    dm.set_grads(3)
    dm.step_transition(3, new, stats=True)
    torch.cuda.synchronize()
    gs = dm.ctx.stats(16, dm.stream)
    for l in range(16):
        s = oracle.step_transition(th_ref[l], dm.host_grad(l), st_ref[l], *new[l], **w.hparams, t=3, want_stats=True)
        assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"{w.name} tensor {l} {old[l]}->{new[l]}")
        assert_stats_close(gs[l], s, f"{w.name} tensor {l}")
    dm.set_grads(4)
    dm.step(4)
    torch.cuda.synchronize()
    for l in range(16):
        oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=4)
        assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"{w.name} after, tensor {l}")


@pytest.mark.parametrize("b_new", [2, 3, 4, 5, 6, 7, 8])
def test_second_moments_exactly_on_thresholds_and_levels(oracle, ctx, b_new):
    # Injected through a 32-bit state: with beta2 = 1/2 and zero gradients the new second moment is exactly
    # half the stored one, so values 2*T_b[k] land exactly on the decision thresholds of a block of scale 1
    # (ties must take the larger level), 2*L_b[c] exactly on the levels, and their fp32 neighbours just
    # beside them.  The first moment does the same for the only exact tie of the linear quantizer (2 bits).
    K = 64
    T = np.array(stq.table(3, b_new), np.float32)
    Lv = np.array(stq.table(2, b_new), np.float32)
    base = np.concatenate([T, np.nextafter(T, np.float32(2)), np.nextafter(T, np.float32(0)), Lv,
                           np.nextafter(Lv, np.float32(0))]).astype(np.float32)
    rows = []
    for i in range(0, base.size, K - 1):       # every block holds one element at the block maximum 1
        blk = np.concatenate([[np.float32(1.0)], base[i:i + K - 1]])
        rows.append(np.pad(blk, (0, K - blk.size), constant_values=np.float32(2.0 ** -20)))
    v_half = np.concatenate(rows).astype(np.float32)
    n = v_half.size
    m_half = np.tile(np.array([1.0, 0.5, -0.5, 0.25, -1.0, 0.0, 0.5, -0.5], np.float32), n // 8 + 1)[:n]
    w = configs.Workload(120 + b_new, f"ties-{b_new}", [("a", n)], K, "fp32", 1, "normal")
    w.hparams.update(beta1=0.5, beta2=0.5)
    dm = DeviceModel(ctx, w, [(32, 32)])
    st = oracle.State.zeros(n, K, 32, 32)
    st.mw[:], st.vw[:] = 2 * m_half, 2 * v_half
    dm.m_codes[0].copy_(torch.from_numpy(oracle.pack_wide(st.mw, 32).view(np.int32)))
    dm.v_codes[0].copy_(torch.from_numpy(oracle.pack_wide(st.vw, 32).view(np.int32)))
    dm.grad[0].zero_()
    th = dm.param[0].cpu().numpy().copy()
    dm.step_transition(1, [(2, b_new)])
    torch.cuda.synchronize()
    oracle.step_transition(th, np.zeros(n, np.float32), st, 2, b_new, **w.hparams, t=1)
    assert_tensor_parity(oracle, dm, 0, th, st, f"ties b={b_new}")
    # the cases really are what they claim: an element on threshold k gets level k (code 2^b-1-k)
    kmax = 2 ** b_new - 1
    on_thr = st.cv.reshape(-1, K)[0, 1:1 + min(K - 1, T.size)]
    assert np.array_equal(on_thr, (kmax - np.arange(on_thr.size)).astype(np.uint8))
    assert np.all(st.sv == 1.0) and np.all(st.sm == 1.0)
    assert set(st.um.tolist()) <= {0, 1, 2} and np.all(st.um[m_half == 0.5] == 1) and np.all(st.um[m_half == -0.5] == 1)


def test_repack_rejects_wide_widths(ctx):
    n = 4096
    cb, _ = stq.state_bytes(n, 128, 32)
    a = torch.zeros(cb // 4, dtype=torch.int32, device="cuda")
    b = torch.zeros(cb // 4, dtype=torch.int32, device="cuda")
    lib = stq.load_library()
    assert lib.stq_repack(ctx._h, n, 128, 0, a.data_ptr(), 16, b.data_ptr(), 8, None) == -3
    assert lib.stq_repack(ctx._h, n, 128, 1, a.data_ptr(), 8, b.data_ptr(), 32, None) == -3
    assert stq.state_bytes(n, 128, 16)[0] == 2 * 64 * 16 * 4 and stq.state_bytes(n, 128, 32)[0] == 2 * 64 * 32 * 4


@pytest.mark.parametrize("tickets,kind", [(False, True), (True, "grad"), (True, True)])
def test_many_small_tensors_in_one_launch(oracle, tickets, kind):
    # 1500 tensors of 1..5000 elements: every wave walks over many tensor boundaries and ragged tiles;
    # with the ticket schedule every ticket of eight neighbouring tiles spans several tensors
    rng = np.random.default_rng(77)
    L = 1500
    tensors = [(f"t{i}", int(rng.integers(1, 5001))) for i in range(L)]
    plan = [(int(rng.integers(2, 9)), int(rng.integers(2, 9))) for _ in range(L)]
    w = configs.Workload(130, "many", tensors, 128, "bf16", 2, "normal_per_tensor")
    c = stq.Context(0, L)
    if tickets:
        c.set_schedule(1)
    dm = DeviceModel(c, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    for t in (1, 2):
        dm.set_grads(t)
        dm.step(t, stats=kind if t == 2 else False)
        torch.cuda.synchronize()
        gs = c.stats(L, dm.stream) if t == 2 else None
        for l in range(L):
            s = oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t, want_stats=True)
            if gs is not None and (l % 13 == 0 or tickets):
                if kind == "grad":   # the gradient's statistics only
                    assert abs(gs[l].g_sq_sum - s.g_sq_sum) <= 1e-12 * s.g_sq_sum and gs[l].g_absmax == s.g_absmax, l
                    assert abs(gs[l].g_abs_sum - s.g_abs_sum) <= 1e-12 * s.g_abs_sum, l
                    assert abs(gs[l].g_sum - s.g_sum) <= 1e-12 * s.g_abs_sum, l
                else:
                    assert_stats_close(gs[l], s, f"many tensor {l}")
    for l in range(L):
        assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"many tensor {l}")
    assert all(gs[l].count == tensors[l][1] for l in range(L))
    c.close()


# ---------------------------------------------------------------- seeded random workloads
@pytest.fixture
def ticket_ctx(ctx):
    """The shared context with the ticket schedule forced for every launch, however small."""
    ctx.set_schedule(1)
    yield ctx
    ctx.set_schedule(0)


@pytest.mark.parametrize("seed", range(12))
def test_random_workloads_ticket_schedule(oracle, ticket_ctx, seed):
    test_random_workloads(oracle, ticket_ctx, seed, grad_stats_only=True)   # every other statistics step: all of them


@pytest.mark.parametrize("seed", range(12))
def test_random_workloads(oracle, ctx, seed, grad_stats_only=False):
    # tensor counts, sizes, block size, gradient type and distribution, widths (quantized and wide),
    # weight decay and the step at which the widths change are all drawn from the seed
    rng = np.random.default_rng(1000 + seed)
    K = int(rng.choice([64, 128, 256]))
    dtype = str(rng.choice(["fp32", "bf16"]))
    kind = str(rng.choice(["normal", "normal_per_tensor", "student_t", "normal_per_tensor_step"]))
    L = int(rng.integers(1, 9))
    tensors = [(f"t{i}", int(rng.choice([1, 17, 2047, 2048, 2049, 3000, 3 * 2048, 5 * 2048 + 99, 20000])) + int(rng.integers(0, 50)))
               for i in range(L)]
    widths = [2, 3, 4, 5, 6, 7, 8] + ([16, 32] if seed % 3 == 0 else [])
    plan = [(int(rng.choice(widths)), int(rng.choice(widths))) for _ in range(L)]
    w = configs.Workload(200 + seed, f"random-{seed}", tensors, K, dtype, 5, kind)
    w.hparams["weight_decay"] = float(rng.choice([0.0, 0.01, 0.1]))
    w.hparams["lr"] = float(rng.choice([1e-4, 1e-3, 3e-2]))
    dm = DeviceModel(ctx, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    switch_at = int(rng.integers(2, 5))
    for t in range(1, 6):
        dm.set_grads(t)
        want_stats = bool(rng.integers(0, 2))
        if want_stats and grad_stats_only and t % 2 == 0:
            want_stats = "grad"
        if t == switch_at:
            new = [(int(rng.choice(widths)), int(rng.choice(widths))) for _ in range(L)]
            dm.step_transition(t, new, stats=want_stats)
        else:
            new = None
            dm.step(t, stats=want_stats)
        torch.cuda.synchronize()
        gs = dm.ctx.stats(L, dm.stream) if want_stats else None
        for l in range(L):
            if new is not None:
                s = oracle.step_transition(th_ref[l], dm.host_grad(l), st_ref[l], *new[l], **w.hparams, t=t, want_stats=True)
            else:
                s = oracle.step(th_ref[l], dm.host_grad(l), st_ref[l], **w.hparams, t=t, want_stats=True)
            assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"{w.name} step {t} tensor {l} {plan[l]}")
            if want_stats == "grad":
                assert gs[l].count == s.count and gs[l].g_absmax == s.g_absmax and gs[l].m_sq_sum == 0
                for name, scale in (("g_sum", s.g_abs_sum), ("g_abs_sum", s.g_abs_sum), ("g_sq_sum", s.g_sq_sum)):
                    assert abs(getattr(gs[l], name) - getattr(s, name)) <= 1e-12 * scale, (t, l, name)
            elif want_stats:
                assert_stats_close(gs[l], s, f"{w.name} step {t} tensor {l}")
        if new is not None:
            plan = new


# --------------------------------------------------------------------- argument checks
def test_argument_checks(ctx):
    w = configs.Workload(94, "args", [("a", 4096)], 128, "fp32", 1, "normal")
    dm = DeviceModel(ctx, w, [(8, 4)])
    lib = stq.load_library()
    import ctypes as C
    hp = hparams(w, 1)

    def call(tensors=dm.tensors, n=1, plan=dm.cplan, hp=hp):
        return lib.stq_step(ctx._h, tensors, n, plan, C.byref(hp), None)

    assert call(plan=binding.make_plan([(9, 4)])) == -3
    assert call(plan=binding.make_plan([(8, 1)])) == -3
    bad = hparams(w, 1); bad.block = 100
    assert call(hp=bad) == -4
    bad = hparams(w, 0)
    assert call(hp=bad) == -1
    for field, value in (("eps", 0.0), ("eps", float("nan")), ("beta1", 1.0), ("beta2", -0.1), ("lr", float("inf")),
                         ("lr", -1e-3), ("weight_decay", float("nan"))):
        bad = hparams(w, 1)
        setattr(bad, field, value)
        assert call(hp=bad) == -1, field
    assert call(n=0) == -1
    t = binding.make_tensors([dict(param=dm.param[0].data_ptr() + 4, grad=dm.grad[0].data_ptr(), numel=4000,
                                   m_codes=dm.m_codes[0].data_ptr(), m_scales=dm.m_scales[0].data_ptr(),
                                   v_codes=dm.v_codes[0].data_ptr(), v_scales=dm.v_scales[0].data_ptr())])
    assert call(tensors=t) == -2
    t = binding.make_tensors([dict(param=None, grad=dm.grad[0].data_ptr(), numel=4000,
                                   m_codes=dm.m_codes[0].data_ptr(), m_scales=dm.m_scales[0].data_ptr(),
                                   v_codes=dm.v_codes[0].data_ptr(), v_scales=dm.v_scales[0].data_ptr())])
    assert call(tensors=t) == -1
    out = (binding.LayerStats * 1)()
    assert lib.stq_stats(ctx._h, out, 1, None) == -7  # nothing accumulated
    torch.cuda.synchronize()


# ------------------------------------------------- the gradient-only statistics flag
@pytest.mark.parametrize("dtype,K", [("fp32", 128), ("bf16", 64)])
def test_gradient_only_statistics_ticket_schedule(oracle, ticket_ctx, dtype, K):
    test_gradient_only_statistics(oracle, ticket_ctx, dtype, K)


@pytest.mark.parametrize("dtype,K", [("fp32", 128), ("bf16", 64)])
def test_gradient_only_statistics(oracle, ctx, dtype, K):
    # STQ_FLAG_STATS_GRAD: the step itself is unchanged, the gradient's sums and maximum agree with the
    # oracle's, the moments' fields stay zero; also across a width-changing step and with ragged tails
    sizes = [3 * 2048 + 5, 2048, 100, 20 * 2048 + 777, 64]
    w = configs.Workload(95, f"gstats-{dtype}", [(f"t{i}", n) for i, n in enumerate(sizes)], K, dtype, 3,
                         "normal_per_tensor")
    plan = [(8, 4), (5, 5), (3, 7), (4, 4), (6, 2)]
    new_plan = [(4, 8), (5, 5), (8, 3), (4, 6), (6, 2)]
    dm = DeviceModel(ctx, w, plan)
    th_ref = [p.cpu().numpy().copy() for p in dm.param]
    st_ref = oracle_states(oracle, w, plan)
    for t in (1, 2, 3):
        dm.set_grads(t)
        if t == 2:
            dm.step_transition(t, new_plan, stats="grad")
        else:
            dm.step(t, stats="grad")
        torch.cuda.synchronize()
        got = dm.ctx.stats(len(sizes), dm.stream)
        for l in range(len(sizes)):
            bm, bv = new_plan[l] if t >= 2 else plan[l]
            s = oracle.step_transition(th_ref[l], dm.host_grad(l), st_ref[l], bm, bv, **w.hparams, t=t, want_stats=True)
            assert_tensor_parity(oracle, dm, l, th_ref[l], st_ref[l], f"gstats step {t}")
            g = got[l]
            assert g.count == s.count
            for name, scale in (("g_sum", s.g_abs_sum), ("g_abs_sum", s.g_abs_sum), ("g_sq_sum", s.g_sq_sum)):
                assert abs(getattr(g, name) - getattr(s, name)) <= 1e-12 * scale, (t, l, name)
            assert g.g_absmax == s.g_absmax
            for name in ("m_sum", "m_sq_sum", "m_err_sq", "m_absmax", "v_sum", "v_sq_sum", "v_err_sq", "v_absmax"):
                assert getattr(g, name) == 0, (t, l, name)


# ------------------------------------------------- statistics of the gradients alone
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_grad_stats_pass(oracle, ctx, dtype):
    # stq_grad_stats: one pass over the gradients, no step; against the oracle's gradient statistics,
    # ragged tails, a one-element tensor, several tiles per wave; accumulates over two calls
    sizes = [1, 63, 2048, 2049, 5 * 2048 + 1000, 300_000, 64]
    w = configs.Workload(96, f"gpass-{dtype}", [(f"t{i}", n) for i, n in enumerate(sizes)], 128, dtype, 2,
                         "normal_per_tensor")
    dm = DeviceModel(ctx, w, [(4, 4)] * len(sizes))
    before = [p.clone() for p in dm.param]
    want = [oracle.Stats() for _ in sizes]
    for t in (1, 2):
        dm.set_grads(t)
        dm.ctx.grad_stats(dm.tensors, w.K, 1 if dtype == "bf16" else 0, dm.stream)
        for l in range(len(sizes)):
            s = oracle.grad_stats(dm.host_grad(l))
            want[l].count += s.count
            want[l].g_sum += s.g_sum; want[l].g_abs_sum += s.g_abs_sum; want[l].g_sq_sum += s.g_sq_sum
            want[l].g_absmax = max(want[l].g_absmax, s.g_absmax)
    got = dm.ctx.stats(len(sizes), dm.stream)
    for l, (g, s) in enumerate(zip(got, want)):
        assert g.count == s.count
        for name, scale in (("g_sum", s.g_abs_sum), ("g_abs_sum", s.g_abs_sum), ("g_sq_sum", s.g_sq_sum)):
            assert abs(getattr(g, name) - getattr(s, name)) <= 1e-12 * scale, (l, name)
        assert g.g_absmax == s.g_absmax
        assert g.m_sq_sum == 0 and g.v_sq_sum == 0
    for p, q in zip(dm.param, before):   # nothing but the accumulators was touched
        assert torch.equal(p, q)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_grad_stats_pass_shows_non_finite_gradients(oracle, ctx, dtype):
    # the documented way to find an overflowed (loss-scaled) gradient before stepping: after a pass over the
    # gradients the tensor's g_sq_sum is not finite; tensors with finite gradients are not affected
    sizes = [5000, 2048 * 3 + 7, 640]
    w = configs.Workload(95, f"gnonfinite-{dtype}", [(f"t{i}", n) for i, n in enumerate(sizes)], 128, dtype, 1,
                         "normal_per_tensor")
    dm = DeviceModel(ctx, w, [(4, 4)] * len(sizes))
    dm.set_grads(1)
    dm.grad[0][4321] = float("inf")
    dm.grad[1][2048 * 3 + 6] = float("nan")
    dm.ctx.grad_stats(dm.tensors, w.K, 1 if dtype == "bf16" else 0, dm.stream)
    got = dm.ctx.stats(len(sizes), dm.stream)
    want = [oracle.grad_stats(dm.host_grad(l)) for l in range(len(sizes))]
    assert not np.isfinite(got[0].g_sq_sum) and not np.isfinite(want[0].g_sq_sum)
    assert got[0].g_absmax == float("inf") == want[0].g_absmax
    assert not np.isfinite(got[1].g_sq_sum) and not np.isfinite(want[1].g_sq_sum)
    assert np.isfinite(got[2].g_sq_sum) and abs(got[2].g_sq_sum - want[2].g_sq_sum) <= 1e-12 * want[2].g_sq_sum


# ------------------------------------------ every statistic under the ticket schedule
# (records of all thirteen values per wave and ticket; the launches here are small, so the schedule is forced)
def test_degenerate_values_ticket_schedule(oracle, ticket_ctx):
    test_degenerate_values(oracle, ticket_ctx)


@pytest.mark.parametrize("dtype,K", [("bf16", 64), ("fp32", 256)])
def test_step_transition_every_width_pair_ticket_schedule(oracle, ticket_ctx, dtype, K):
    test_step_transition_every_width_pair(oracle, ticket_ctx, dtype, K)


@pytest.mark.parametrize("dtype,K", [("fp32", 128), ("bf16", 64)])
def test_wide_states_every_combination_ticket_schedule(oracle, ticket_ctx, dtype, K):
    test_wide_states_every_combination(oracle, ticket_ctx, dtype, K)


@pytest.mark.parametrize("dtype,K", [("bf16", 128)])
def test_transitions_among_the_papers_widths_ticket_schedule(oracle, ticket_ctx, dtype, K):
    test_transitions_among_the_papers_widths(oracle, ticket_ctx, dtype, K)
