"""Pins of the oracle's Adam step (Alg. 1 inner loop): closed forms, the textbook AdamW
it reduces to when quantization is exact, invariants of the quantized update, statistics."""
import numpy as np
import pytest
import torch

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)


def test_first_step_closed_form(oracle):
    # blocks of one element quantize exactly (the element is its own block maximum), so from
    # m0 = v0 = 0:  m~ = g, v~ = g^2  and  dtheta = -lr * g / (|g| + eps) - lr*wd*theta
    g = np.array([3e-4, -2.0, 1e-7, 5.0, -1e-3], np.float32)
    th0 = np.array([0.5, -0.25, 0.125, 1.0, -2.0], np.float32)
    for wd in (0.0, 0.1):
        th = th0.copy()
        st = oracle.State.zeros(g.size, 1, 8, 4)
        oracle.step(th, g, st, **{**HP, "weight_decay": wd}, t=1)
        g64, t64 = g.astype(np.float64), th0.astype(np.float64)
        want = t64 * (1 - 1e-3 * wd) - 1e-3 * g64 / (np.abs(g64) + 1e-8)
        np.testing.assert_allclose(th, want, rtol=2e-6, atol=0)
        # with eps negligible the step is -lr*sign(g)
        np.testing.assert_allclose((th - th0 * np.float32(1 - 1e-3 * wd))[[0, 1, 3, 4]],
                                   -1e-3 * np.sign(g[[0, 1, 3, 4]]), rtol=1e-3)


def test_constant_gradient_keeps_unit_ratio(oracle):
    # constant g with exact (K=1) quantization: m~_t = g and v~_t = g^2 for every t
    g = np.array([2e-3, -7e-5], np.float32)
    th = np.zeros(2, np.float32)
    st = oracle.State.zeros(2, 1, 8, 8)
    for t in range(1, 31):
        before = th.copy()
        oracle.step(th, g, st, **HP, t=t)
        np.testing.assert_allclose(th - before, -1e-3 * np.sign(g), rtol=2e-3)


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_reduces_to_textbook_adamw_when_quantization_is_exact(oracle, wd):
    # K=1: every element is its block's maximum -> top code, dequantizes to itself.  The oracle
    # must then follow decoupled-weight-decay Adam; torch.optim.AdamW is the library routine.
    rng = np.random.default_rng(11)
    n = 257
    th0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    th = th0.copy()
    st = oracle.State.zeros(n, 1, 5, 3)
    p = torch.nn.Parameter(torch.tensor(th0.astype(np.float64)))
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(float(np.float32(0.9)), float(np.float32(0.999))),
                            eps=float(np.float32(1e-8)), weight_decay=wd)
    for t in range(1, 26):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        oracle.step(th, g, st, **{**HP, "weight_decay": wd}, t=t)
        p.grad = torch.tensor(g.astype(np.float64))
        opt.step()
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=0, atol=3e-6)
    # and the stored moments are the exact Adam moments
    m = st.sm * np.array([oracle.R(5, int(u)) for u in st.um], np.float32)
    np.testing.assert_allclose(m, opt.state[p]["exp_avg"].numpy(), rtol=1e-5, atol=1e-10)  # fp32 accumulation vs float64
    np.testing.assert_allclose(st.sv, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-5)


@pytest.mark.parametrize("K,bm,bv", [(128, 8, 4), (64, 4, 3), (256, 6, 4), (128, 2, 2), (128, 5, 8)])
def test_update_uses_the_requantized_moments(oracle, K, bm, bv):
    # Alg. 1: the bias correction and the parameter update read \hat m_t, \hat v_t (the quantized
    # values), so theta' must be a function of the NEW stored state only.
    rng = np.random.default_rng(K + bm)
    n = 3 * K + 17  # ragged last block
    th0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    st = oracle.State.zeros(n, K, bm, bv)
    th = th0.copy()
    for t in range(1, 4):
        prev = th.copy()
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        oracle.step(th, g, st, **HP, t=t)
        blk = np.arange(n) // K
        mq = st.sm[blk].astype(np.float64) * np.array([oracle.R(bm, int(u)) for u in st.um], np.float64)
        vq = st.sv[blk].astype(np.float64) * np.array([oracle.Lv(bv, int(c)) for c in st.cv], np.float64)
        want = prev - 1e-3 * (mq / (1 - 0.9 ** t)) / (np.sqrt(vq / (1 - 0.999 ** t)) + 1e-8)
        np.testing.assert_allclose(th, want, rtol=0, atol=2e-6 * 1e-3 * 40 + 1e-9)
        # quantization really happened (it is not the unquantized Adam)
        assert len(np.unique(st.um)) <= 2 ** bm - 1 and st.um.max() <= 2 ** bm - 2
        assert np.all(vq > 0)


def test_blocks_are_independent(oracle):
    rng = np.random.default_rng(5)
    K, n = 128, 128 * 6
    th = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    st = oracle.State.zeros(n, K, 6, 4)
    full_th = th.copy()
    oracle.step(full_th, g, st, **HP, t=1)
    # the same blocks processed alone give the same result
    for j in (0, 3, 5):
        sl = slice(j * K, (j + 1) * K)
        sub = oracle.State.zeros(K, K, 6, 4)
        sub_th = th[sl].copy()
        oracle.step(sub_th, g[sl].copy(), sub, **HP, t=1)
        assert np.array_equal(sub_th, full_th[sl])
        assert np.array_equal(sub.um, st.um[sl]) and sub.sm[0] == st.sm[j]
        assert np.array_equal(sub.cv, st.cv[sl]) and sub.sv[0] == st.sv[j]


def test_bf16_gradients_are_widened_exactly(oracle):
    rng = np.random.default_rng(9)
    n = 300
    g32 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    gb = (g32.view(np.uint32) >> 16).astype(np.uint16)           # bf16 bit patterns (truncated)
    gw = (gb.astype(np.uint32) << 16).view(np.float32)           # the fp32 values they denote
    th_a = (rng.standard_normal(n) * 0.02).astype(np.float32)
    th_b = th_a.copy()
    sa, sb = oracle.State.zeros(n, 64, 8, 4), oracle.State.zeros(n, 64, 8, 4)
    oracle.step(th_a, gb, sa, **HP, t=1)
    oracle.step(th_b, gw, sb, **HP, t=1)
    assert np.array_equal(th_a, th_b) and np.array_equal(sa.um, sb.um) and np.array_equal(sa.cv, sb.cv)


def test_statistics_match_float64_numpy(oracle):
    rng = np.random.default_rng(21)
    n, K = 1000, 128
    th = (rng.standard_normal(n) * 0.02).astype(np.float32)
    st = oracle.State.zeros(n, K, 8, 4)
    oracle.step(th, (rng.standard_normal(n) * 1e-3).astype(np.float32), st, **HP, t=1)
    prev = st.copy()
    g = (rng.standard_normal(n) * 2e-3).astype(np.float32)
    s = oracle.step(th, g, st, **HP, t=2, want_stats=True)
    blk = np.arange(n) // K
    mh = prev.sm[blk] * np.array([oracle.R(8, int(u)) for u in prev.um], np.float32)
    vh = prev.sv[blk] * np.array([oracle.Lv(4, int(c)) for c in prev.cv], np.float32)
    m = np.float32(0.9) * mh + (np.float32(1) - np.float32(0.9)) * g
    v = np.float32(0.999) * vh + (np.float32(1) - np.float32(0.999)) * (g * g)
    mq = st.sm[blk] * np.array([oracle.R(8, int(u)) for u in st.um], np.float32)
    vq = st.sv[blk] * np.array([oracle.Lv(4, int(c)) for c in st.cv], np.float32)
    g64, m64, v64 = g.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    assert s.count == n
    np.testing.assert_allclose(s.g_sum, g64.sum(), rtol=1e-12)
    np.testing.assert_allclose(s.g_abs_sum, np.abs(g64).sum(), rtol=1e-12)
    np.testing.assert_allclose(s.g_sq_sum, (g64 ** 2).sum(), rtol=1e-12)
    assert s.g_absmax == np.abs(g).max()
    np.testing.assert_allclose(s.m_sum, m64.sum(), rtol=1e-10)
    np.testing.assert_allclose(s.m_sq_sum, (m64 ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(s.m_err_sq, ((m64 - mq) ** 2).sum(), rtol=1e-10)
    assert s.m_absmax == np.abs(m).max() == st.sm.max()
    np.testing.assert_allclose(s.v_sum, v64.sum(), rtol=1e-12)
    np.testing.assert_allclose(s.v_sq_sum, (v64 ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(s.v_err_sq, ((v64 - vq) ** 2).sum(), rtol=1e-10)
    assert s.v_absmax == v.max() == st.sv.max()
    # Eq. 2 / Eq. 8 identity: v_l = n_l^2
    n_l = np.sqrt(s.g_sq_sum / n)
    assert abs(s.g_sq_sum / n - n_l ** 2) < 1e-18


def test_gradient_statistics_show_non_finite_gradients(oracle):
    # the precondition of the step is finite gradients; the gradient pass is how a caller finds out
    g = (np.random.default_rng(3).standard_normal(500) * 1e-3).astype(np.float32)
    assert np.isfinite(oracle.grad_stats(g).g_sq_sum)
    for bad in (np.inf, -np.inf, np.nan):
        h = g.copy()
        h[123] = bad
        s = oracle.grad_stats(h)
        assert not np.isfinite(s.g_sq_sum)
        if np.isinf(bad):
            assert s.g_absmax == np.inf
    # bf16 bit patterns: 0x7F80 = +Inf, 0x7FC0 = NaN
    hb = np.zeros(64, np.uint16)
    hb[5] = 0x7F80
    assert oracle.grad_stats(hb).g_sq_sum == np.inf
    hb[5] = 0x7FC0
    assert np.isnan(oracle.grad_stats(hb).g_sq_sum)
