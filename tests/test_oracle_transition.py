"""Pins of the oracle's width-changing step (Algorithm 1 maps the layer's new width before the
layer loop, so that step reads the stored moments at the old width and quantizes at the new one)."""
import numpy as np
import pytest

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def _rand_state(oracle, rng, n, K, bm, bv):
    st = oracle.State.zeros(n, K, bm, bv)
    th = rng.normal(0, 0.02, n).astype(np.float32)
    for t in (1, 2):
        oracle.step(th, rng.normal(0, 1e-3, n).astype(np.float32), st, **HP, t=t)
    return th, st


@pytest.mark.parametrize("widths", [(8, 4, 8, 4), (3, 6, 3, 6)])
def test_same_widths_is_the_plain_step(oracle, widths):
    rng = np.random.default_rng(1)
    bm, bv, _, _ = widths
    th, st = _rand_state(oracle, rng, 1000, 128, bm, bv)
    g = rng.normal(0, 1e-3, 1000).astype(np.float32)
    th2, st2 = th.copy(), st.copy()
    oracle.step(th, g, st, **HP, t=3)
    oracle.step_transition(th2, g, st2, bm, bv, **HP, t=3)
    assert np.array_equal(th.view(np.uint32), th2.view(np.uint32))
    assert np.array_equal(st.um, st2.um) and np.array_equal(st.cv, st2.cv)
    assert np.array_equal(st.sm, st2.sm) and np.array_equal(st.sv, st2.sv)


@pytest.mark.parametrize("new", [(2, 2), (4, 8), (8, 3)])
def test_from_the_zero_state_only_the_new_widths_matter(oracle, new):
    # m_0 = v_0 = 0 dequantizes to 0 at every width, so a first step that changes widths equals a
    # plain first step at the new widths
    rng = np.random.default_rng(2)
    n = 700
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    a, b = th0.copy(), th0.copy()
    sa = oracle.State.zeros(n, 64, 5, 6)
    sb = oracle.State.zeros(n, 64, *new)
    oracle.step_transition(a, g, sa, *new, **HP, t=1)
    oracle.step(b, g, sb, **HP, t=1)
    assert (sa.bm, sa.bv) == new
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(sa.um, sb.um) and np.array_equal(sa.cv, sb.cv)
    assert np.array_equal(sa.sm, sb.sm) and np.array_equal(sa.sv, sb.sv)


@pytest.mark.parametrize("old,new", [((8, 4), (4, 8)), ((3, 3), (6, 5)), ((6, 8), (2, 2)), ((5, 2), (5, 7))])
def test_reads_old_width_writes_new_width(oracle, old, new):
    # the composition written out with the separately pinned block quantizers: dequantize the stored
    # codes at the OLD widths, Adam moment update in separately rounded fp32, quantize at the NEW widths
    rng = np.random.default_rng(3)
    n, K = 5 * 128 + 37, 128
    th, st = _rand_state(oracle, rng, n, K, *old)
    g = rng.normal(0, 2e-3, n).astype(np.float32)
    um0, cv0, sm0, sv0 = st.um.copy(), st.cv.copy(), st.sm.copy(), st.sv.copy()
    oracle.step_transition(th, g, st, *new, **HP, t=3)
    b1, b2 = np.float32(HP["beta1"]), np.float32(HP["beta2"])
    for j in range((n + K - 1) // K):
        sl = slice(j * K, min(n, (j + 1) * K))
        mh = oracle.dequant_linear_block(um0[sl], old[0], sm0[j])
        vh = oracle.dequant_log_block(cv0[sl], old[1], sv0[j])
        m = (b1 * mh).astype(np.float32) + ((np.float32(1) - b1) * g[sl]).astype(np.float32)
        v = (b2 * vh).astype(np.float32) + ((np.float32(1) - b2) * (g[sl] * g[sl]).astype(np.float32)).astype(np.float32)
        um, s_m = oracle.quant_linear_block(m.astype(np.float32), new[0])
        cv, s_v = oracle.quant_log_block(v.astype(np.float32), new[1])
        assert np.array_equal(um, st.um[sl]) and np.array_equal(cv, st.cv[sl]), j
        assert s_m == st.sm[j] and s_v == st.sv[j]
        assert st.um[sl].max() <= 2 ** new[0] - 2 and st.cv[sl].max() <= 2 ** new[1] - 1


def test_widening_v_alone_changes_nothing_it_need_not(oracle):
    # the log grids are nested: reading v at 3 bits and writing at 6 bits must give the same new
    # second moment values as first re-packing 3 -> 6 bits (lossless) and then stepping at 6 bits
    rng = np.random.default_rng(4)
    n, K = 900, 64
    th, st = _rand_state(oracle, rng, n, K, 8, 3)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    a, sa = th.copy(), st.copy()
    b, sb = th.copy(), st.copy()
    oracle.step_transition(a, g, sa, 8, 6, **HP, t=3)
    sb.cv, sb.bv = oracle.repack(sb.cv, 1, 3, 6), 6
    oracle.step(b, g, sb, **HP, t=3)
    assert np.array_equal(sa.cv, sb.cv) and np.array_equal(sa.sv, sb.sv)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
