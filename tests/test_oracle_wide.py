"""Pins of the oracle's wide states: the paper's width set B = {4, 8, 16, 32} has two members that are
not block-quantized.  32 bits keeps the fp32 value (the step is then plain AdamW), 16 bits its bfloat16
rounding."""
import numpy as np
import pytest
import torch

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def test_bfloat16_rounding_matches_torch(oracle):
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.uniform(-30, 30, 2000),
                        [0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e-39, 1.0e-45]]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.wide_value(v, 16) for v in x], np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.wide_value(1.00390625, 16) == 1.0 and oracle.wide_value(1.01171875, 16) == 1.015625
    assert all(oracle.wide_value(float(v), 32) == float(v) for v in x[:50])


def test_32_bit_states_are_textbook_adamw(oracle):
    # nothing is quantized at 32 bits: the step is AdamW in fp32 with the same operation order
    rng = np.random.default_rng(1)
    n = 3000
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    th = th0.copy()
    st = oracle.State.zeros(n, 128, 32, 32)
    p = torch.nn.Parameter(torch.from_numpy(th0.copy()).double())
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"], weight_decay=HP["weight_decay"])
    for t in range(1, 21):
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        oracle.step(th, g, st, **HP, t=t)
        p.grad = torch.from_numpy(g).double()
        opt.step()
    ref = p.detach().numpy()
    assert np.max(np.abs(th - ref) / np.maximum(np.abs(ref), 1e-3)) < 2e-5
    # and the stored moments are the exact recurrences in separately rounded fp32
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    rng = np.random.default_rng(1); rng.normal(0, 0.02, n)
    b1, b2 = np.float32(0.9), np.float32(0.999)
    for t in range(1, 21):
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        m = (b1 * m).astype(np.float32) + ((np.float32(1) - b1) * g).astype(np.float32)
        v = (b2 * v).astype(np.float32) + ((np.float32(1) - b2) * (g * g).astype(np.float32)).astype(np.float32)
    assert np.array_equal(st.mw, m) and np.array_equal(st.vw, v)


def test_16_bit_states_hold_bfloat16_values(oracle):
    rng = np.random.default_rng(2)
    n = 1500
    th = rng.normal(0, 0.02, n).astype(np.float32)
    st = oracle.State.zeros(n, 64, 16, 16)
    for t in range(1, 6):
        s = oracle.step(th, rng.normal(0, 1e-3, n).astype(np.float32), st, **HP, t=t, want_stats=True)
    for arr in (st.mw, st.vw):
        assert np.all(arr.view(np.uint32) & 0xFFFF == 0)          # representable in bfloat16
    assert np.all(st.vw >= 0)
    # the recorded quantization error is that of the bfloat16 rounding: relative 2^-9 at most
    assert 0 < s.m_err_sq <= s.m_sq_sum * 2.0 ** -18 and 0 < s.v_err_sq <= s.v_sq_sum * 2.0 ** -18


@pytest.mark.parametrize("old,new", [((16, 16), (4, 4)), ((8, 4), (32, 16)), ((32, 32), (16, 8)), ((4, 16), (16, 4))])
def test_transitions_between_wide_and_quantized(oracle, old, new):
    # written out with the separately pinned pieces: the stored value at the old width, the fp32 moment
    # update, then either the block quantizer or the wide rounding at the new width
    rng = np.random.default_rng(3)
    n, K = 3 * 128 + 50, 128
    th = rng.normal(0, 0.02, n).astype(np.float32)
    st = oracle.State.zeros(n, K, *old)
    for t in (1, 2):
        oracle.step(th, rng.normal(0, 1e-3, n).astype(np.float32), st, **HP, t=t)
    g = rng.normal(0, 2e-3, n).astype(np.float32)
    before = st.copy()
    oracle.step_transition(th, g, st, *new, **HP, t=3)
    assert (st.bm, st.bv) == new
    b1, b2 = np.float32(HP["beta1"]), np.float32(HP["beta2"])
    for j in range((n + K - 1) // K):
        sl = slice(j * K, min(n, (j + 1) * K))
        mh = before.mw[sl] if old[0] >= 16 else oracle.dequant_linear_block(before.um[sl], old[0], before.sm[j])
        vh = before.vw[sl] if old[1] >= 16 else oracle.dequant_log_block(before.cv[sl], old[1], before.sv[j])
        m = ((b1 * mh).astype(np.float32) + ((np.float32(1) - b1) * g[sl]).astype(np.float32)).astype(np.float32)
        v = ((b2 * vh).astype(np.float32) + ((np.float32(1) - b2) * (g[sl] * g[sl]).astype(np.float32)).astype(np.float32)).astype(np.float32)
        if new[0] >= 16:
            want = np.array([oracle.wide_value(x, new[0]) for x in m], np.float32)
            assert np.array_equal(st.mw[sl].view(np.uint32), want.view(np.uint32))
        else:
            um, s_m = oracle.quant_linear_block(m, new[0])
            assert np.array_equal(um, st.um[sl]) and s_m == st.sm[j]
        if new[1] >= 16:
            want = np.array([oracle.wide_value(x, new[1]) for x in v], np.float32)
            assert np.array_equal(st.vw[sl].view(np.uint32), want.view(np.uint32))
        else:
            cv, s_v = oracle.quant_log_block(v, new[1])
            assert np.array_equal(cv, st.cv[sl]) and s_v == st.sv[j]


@pytest.mark.parametrize("b", [16, 32])
def test_wide_layout_is_the_tile_format_with_wide_codes(oracle, b):
    # element idx = tile*2048 + 256 i + 4 j + e is code n = 4i + e of lane j: for 32 bits word n of the lane,
    # for 16 bits half (n & 1) of word n >> 1; word p of lane j sits at tile*64*b + p*64 + j
    rng = np.random.default_rng(4)
    n = 2048 + 700
    vals = np.array([oracle.wide_value(x, b) for x in rng.standard_normal(n)], np.float32)
    words = oracle.pack_wide(vals, b)
    assert words.size == 2 * 64 * b
    bits = vals.view(np.uint32)
    for idx in rng.integers(0, n, 300):
        tile, r = divmod(int(idx), 2048)
        i, j, e = r // 256, (r % 256) // 4, r % 4
        k = 4 * i + e
        if b == 32:
            assert words[tile * 64 * 32 + k * 64 + j] == bits[idx]
        else:
            w = words[tile * 64 * 16 + (k >> 1) * 64 + j]
            assert (w >> (16 * (k & 1))) & 0xFFFF == bits[idx] >> 16
    assert np.array_equal(oracle.unpack_wide(words, n, b).view(np.uint32), bits)
    # pad elements are stored as zero bits
    padded = np.concatenate([vals, np.zeros(4096 - n, np.float32)])
    assert np.array_equal(words, oracle.pack_wide(padded, b))
