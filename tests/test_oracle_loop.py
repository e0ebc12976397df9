"""Pins of the oracle's whole iteration (Algorithm 1: layer loop every step, statistics -> EMAs ->
score -> Map when t mod U = 0 or t < 5, the new widths written by the following step)."""
import numpy as np

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
SIZES = (700, 2048 + 300, 128)



def _grads(sizes, sigmas, seed):
    def of_step(t):
        rng = np.random.default_rng(seed + 1009 * t)
        return [rng.normal(0, s, n).astype(np.float32) for n, s in zip(sizes, sigmas)]
    return of_step


def test_with_a_single_width_the_loop_is_the_plain_step_repeated(oracle):
    rng = np.random.default_rng(0)
    K = 128
    params = [rng.normal(0, 0.02, n).astype(np.float32) for n in SIZES]
    ref = [p.copy() for p in params]
    states = [oracle.State.zeros(n, K, 6, 6) for n in SIZES]
    ref_states = [oracle.State.zeros(n, K, 6, 6) for n in SIZES]
    grads = _grads(SIZES, (1e-3, 1e-4, 1e-2), 5)
    log, nxt, _ = oracle.loop(params, states, grads, 7, 3, HP, dict(thr=(), bits=(6,), alpha=0.3, tau=10.0))
    for t in range(1, 8):
        for p, g, st in zip(ref, grads(t), ref_states):
            oracle.step(p, g, st, **HP, t=t)
    for p, q, a, b in zip(params, ref, states, ref_states):
        assert np.array_equal(p.view(np.uint32), q.view(np.uint32))
        assert np.array_equal(a.um, b.um) and np.array_equal(a.cv, b.cv)
        assert np.array_equal(a.sm, b.sm) and np.array_equal(a.sv, b.sv)
    assert nxt == [(6, 6)] * 3


def test_cadence_and_one_step_delay(oracle):
    # decisions at t = 1..4 and at multiples of U; the widths written at step t are the ones mapped
    # from the last decision before t (Map: width = bits[#thresholds <= score]; the paper's ladder)
    rng = np.random.default_rng(1)
    K, U = 64, 6
    thr, bits = (6.8, 12.0, 24.0), (4, 8, 16, 32)
    params = [rng.normal(0, 0.02, n).astype(np.float32) for n in SIZES]
    states = [oracle.State.zeros(n, K, 16, 16) for n in SIZES]   # the paper's initial width
    log, nxt, ema = oracle.loop(params, states, _grads(SIZES, (3e-2, 1e-3, 1e-5), 7), 13, U, HP,
                                dict(thr=thr, bits=bits, alpha=0.5, tau=5.0))
    due = [t for t, _, sc in log if sc is not None]
    assert due == [1, 2, 3, 4, 6, 12]
    expect = [(16, 16)] * 3
    for t, written, sc in log:
        assert written == expect, t
        if sc is not None:
            expect = [(bits[sum(x <= s for x in thr)],) * 2 for s in sc]
    assert nxt == expect
    assert [(st.bm, st.bv) for st in states] == log[-1][1]
    # layers with larger gradients score higher (both ratios of Eq. 2 and Eq. 8 grow with the scale)
    sc = log[0][2]
    assert sc[0] > sc[1] > sc[2]
    assert ema.n_ema > 0 and ema.v_ema > 0


def test_first_decision_from_equal_layers_gives_phi_plus_log2_S(oracle):
    # identical layers: every ratio to the (first) EMA is 1/alpha, so with alpha = 1 the score is
    # phi + log2 S_1 for every layer
    K = 128
    g = np.random.default_rng(3).normal(0, 1e-3, 512).astype(np.float32)
    params = [np.zeros(512, np.float32) for _ in range(3)]
    states = [oracle.State.zeros(512, K, 8, 8) for _ in range(3)]
    log, _, _ = oracle.loop(params, states, lambda t: [g, g, g], 1, 0, HP,
                            dict(alpha=1.0, tau=4.0, eps=0.0))
    want = 7.2 + np.log2(1.0 + 1.0 / np.cosh(1.0 / 4.0))
    assert np.allclose(log[0][2], want, rtol=0, atol=1e-12)


def test_loop_can_be_resumed_step_by_step(oracle):
    # one call over 8 steps == eight calls of one step that hand on the EMAs and the pending widths
    K, U = 128, 3
    kw = dict(thr=(5.0, 7.5, 10.0), bits=(3, 4, 6, 8), alpha=0.3, tau=4.0, v_offset=-0.5)
    grads = _grads(SIZES, (1e-2, 1e-3, 1e-5), 9)
    runs = []
    for split in (False, True):
        rng = np.random.default_rng(2)
        params = [rng.normal(0, 0.02, n).astype(np.float32) for n in SIZES]
        states = [oracle.State.zeros(n, K, 8, 8) for n in SIZES]
        if not split:
            log, nxt, ema = oracle.loop(params, states, grads, 8, U, HP, kw)
        else:
            log, nxt, ema = [], None, None
            for t in range(1, 9):
                lg, nxt, ema = oracle.loop(params, states, grads, 1, U, HP, kw, ema=ema, first_step=t, next_plan=nxt)
                log += lg
        runs.append((params, states, [w for _, w, _ in log], nxt, (ema.n_ema, ema.r_ema, ema.v_ema)))
    a, b = runs
    assert a[2] == b[2] and a[3] == b[3] and a[4] == b[4]
    assert len({tuple(w) for w in a[2]}) > 2   # widths really change along the way
    for p, q, s, r in zip(a[0], b[0], a[1], b[1]):
        assert np.array_equal(p.view(np.uint32), q.view(np.uint32))
        assert np.array_equal(s.um, r.um) and np.array_equal(s.cv, r.cv)


def test_gradient_statistics_alone(oracle):
    # against numpy float64, fp32 and bf16 gradients; equal to the statistics the step gathers
    rng = np.random.default_rng(4)
    g = (rng.standard_t(3, 5000) * 1e-3).astype(np.float32)
    s = oracle.grad_stats(g)
    g64 = g.astype(np.float64)
    assert s.count == 5000 and s.g_absmax == np.abs(g).max()
    assert np.isclose(s.g_sum, g64.sum(), rtol=1e-12, atol=1e-18)
    assert np.isclose(s.g_abs_sum, np.abs(g64).sum(), rtol=1e-12) and np.isclose(s.g_sq_sum, (g64 * g64).sum(), rtol=1e-12)
    hb = (g.view(np.uint32) >> 16).astype(np.uint16)          # truncation to bf16 is good enough here
    sb = oracle.grad_stats(hb)
    gb = (hb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.isclose(sb.g_abs_sum, np.abs(gb).sum(), rtol=1e-12) and sb.g_absmax == np.abs(gb).max()
    st = oracle.State.zeros(5000, 128, 6, 6)
    via_step = oracle.step(np.zeros(5000, np.float32), g, st, **HP, t=1, want_stats=True)
    got = (via_step.g_sum, via_step.g_abs_sum, via_step.g_sq_sum, via_step.g_absmax, via_step.count)
    assert got == (s.g_sum, s.g_abs_sum, s.g_sq_sum, s.g_absmax, s.count)


def test_algorithm1_order_applies_the_decision_in_the_same_step(oracle):
    # the written order: Map before the layer loop.  Its plan at step t is what the by-product order
    # (statistics gathered during the step) writes one step later, as long as both see the same gradients
    # and EMAs -- so with gradients that do not depend on the state the two logs are shifted copies.
    K, U = 64, 5
    kw = dict(thr=(5.0, 7.5, 10.0), bits=(3, 4, 6, 8), alpha=0.3, tau=4.0, v_offset=-0.5)
    grads = _grads(SIZES, (1e-2, 1e-3, 1e-5), 21)
    out = []
    for fn in (oracle.loop_alg1_order, oracle.loop):
        rng = np.random.default_rng(6)
        params = [rng.normal(0, 0.02, n).astype(np.float32) for n in SIZES]
        states = [oracle.State.zeros(n, K, 8, 8) for n in SIZES]
        res = fn(params, states, grads, 11, U, HP, kw)
        out.append((res[0], params, states))
    alg1, delayed = out[0][0], out[1][0]
    for (t, plan, sc), (_, _, sc_d) in zip(alg1, delayed):
        assert (sc is None) == (sc_d is None)
        if sc is not None:
            assert np.array_equal(sc, sc_d)          # same statistics, same EMAs, same scores
    for k in range(len(alg1) - 1):
        assert alg1[k][1] == delayed[k + 1][1]       # ... applied one step earlier
    assert alg1[0][1] != [(8, 8)] * 3                # step 1 already writes the decided widths
    # and the first step equals a plain first step at those widths (m_0 = v_0 = 0)
    rng = np.random.default_rng(6)
    p0 = [rng.normal(0, 0.02, n).astype(np.float32) for n in SIZES]
    for p, g, (bm, bv) in zip(p0, grads(1), alg1[0][1]):
        oracle.step(p, g, oracle.State.zeros(p.size, K, bm, bv), **HP, t=1)
    rng = np.random.default_rng(6)
    q0 = [rng.normal(0, 0.02, n).astype(np.float32) for n in SIZES]
    st0 = [oracle.State.zeros(n, K, 8, 8) for n in SIZES]
    oracle.loop_alg1_order(q0, st0, grads, 1, U, HP, kw)
    for p, q in zip(p0, q0):
        assert np.array_equal(p.view(np.uint32), q.view(np.uint32))
