"""Pins of the oracle's packed layout, its bit-width transition and its bit-width decision."""
import math
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")
BITS = [2, 3, 4, 5, 6, 7, 8]


def read_constants():
    out = {}
    for line in open(os.path.join(GOLD, "paper_constants.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals = [float(t) for t in v.split()]
            out[k.strip()] = vals[0] if len(vals) == 1 else vals
    return out


# ------------------------------------------------------------------- layout
def bigint_pack(codes, b):
    """Independent packer: one Python big integer per (tile, lane) bit stream."""
    n = len(codes)
    tiles = (n + 2047) // 2048
    words = np.zeros(tiles * 64 * b, np.uint32)
    for tile in range(tiles):
        for j in range(64):
            stream = 0
            for i in range(8):
                for e in range(4):
                    idx = tile * 2048 + 256 * i + 4 * j + e
                    if idx < n:
                        stream |= int(codes[idx]) << ((4 * i + e) * b)
            for p in range(b):
                words[tile * 64 * b + p * 64 + j] = (stream >> (32 * p)) & 0xFFFFFFFF
    return words


def test_layout_hand_placements(oracle):
    n_cases = 0
    for line in open(os.path.join(GOLD, "layout_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        lhs, rhs = line.split("->")
        b, idx = (int(t) for t in lhs.split())
        word, bit = (int(t) for t in rhs.split())
        numel = 4096
        codes = np.zeros(numel, np.uint8)
        codes[idx] = 2 ** b - 1  # all b bits set
        w = oracle.pack(codes, b)
        nz = np.flatnonzero(w)
        lo_bits = min(b, 32 - bit)
        assert w[word] == ((2 ** lo_bits - 1) << bit), line
        if lo_bits < b:  # straddles into the lane's next word, 64 words further on
            assert w[word + 64] == 2 ** (b - lo_bits) - 1, line
            assert set(nz) == {word, word + 64}
        else:
            assert set(nz) == {word}
        n_cases += 1
    assert n_cases == 12


def test_scale_padding_hand_cases(oracle):
    """pad_scales: real entries first and in block order, zeros after, size per the hand cases."""
    n_cases = 0
    for line in open(os.path.join(GOLD, "scale_padding_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        lhs, rhs = line.split("->")
        numel, K = (int(t) for t in lhs.split())
        real, stored = (int(t) for t in rhs.split())
        s = np.arange(1, real + 1, dtype=np.float32)  # every real entry non-zero and distinct
        out = oracle.pad_scales(s, numel, K)
        assert out.dtype == np.float32 and out.size == stored, line
        assert np.array_equal(out[:real], s), line
        assert not out[real:].any(), line
        # the number of real entries is the number of blocks the oracle's state holds
        assert oracle.State.zeros(numel, K, 4, 4).sm.size == real, line
        n_cases += 1
    assert n_cases == 7


@pytest.mark.parametrize("b", BITS)
@pytest.mark.parametrize("numel", [1, 3, 255, 2048, 2049, 5000])
def test_pack_roundtrip_and_independent_packer(oracle, b, numel):
    rng = np.random.default_rng(b * 1000 + numel)
    codes = rng.integers(0, 2 ** b, numel, dtype=np.uint8)
    w = oracle.pack(codes, b)
    assert w.size == ((numel + 2047) // 2048) * 64 * b == oracle.code_words(numel, b)
    assert np.array_equal(w, bigint_pack(codes, b))
    assert np.array_equal(oracle.unpack(w, numel, b), codes)
    # pad elements carry zero bits: total popcount equals that of the real codes
    assert sum(bin(int(x)).count("1") for x in w) == sum(bin(int(x)).count("1") for x in codes)


def test_state_bytes_per_param_matches_paper_scale():
    # layout cost: (bm+bv)/8 + 8/K bytes per parameter.  At the paper's average of 5.1 bits the
    # saving vs 32-bit states (8 B/param) must land near the paper's 84.4 % headline and its
    # GPT2-XL figure 12.00 GB -> 1.86 GB (= 84.5 %).
    c = read_constants()
    per_param = 2 * c["avg_bits"] / 8 + 8 / 128
    saved = 1 - per_param / 8
    paper_saved = 1 - c["gpt2xl_state_gb_stq"] / c["gpt2xl_state_gb_full"]
    assert abs(paper_saved * 100 - c["saved_headline_percent"]) < 0.2
    assert abs(saved - paper_saved) < 0.015
    assert (1 - (2 * 8 / 8) / 8) * 100 == c["saved_8bit_percent"]


# -------------------------------------------------------------------- repack
@pytest.mark.parametrize("b_old", BITS)
@pytest.mark.parametrize("b_new", BITS)
def test_repack_equals_requantizing_the_decoded_block(oracle, b_old, b_new):
    # linear: all codes of the old width, in a block whose maximum is 1 (scale stays 1)
    qo = 2 ** (b_old - 1) - 1
    u = np.arange(0, 2 * qo + 1, dtype=np.uint8)
    x = oracle.dequant_linear_block(u, b_old, 1.0)
    want, s = oracle.quant_linear_block(x, b_new)
    assert s == 1.0
    assert np.array_equal(oracle.repack(u, 0, b_old, b_new), want)
    # log
    c = np.arange(0, 2 ** b_old, dtype=np.uint8)
    y = oracle.dequant_log_block(c, b_old, 1.0)
    want, s = oracle.quant_log_block(y, b_new)
    assert s == 1.0
    got = oracle.repack(c, 1, b_old, b_new)
    assert np.array_equal(got, want)
    if b_new >= b_old:
        # nested grids: widening is lossless wherever the old level is inside the new range
        y2 = oracle.dequant_log_block(got, b_new, 1.0)
        inside = y >= oracle.Lv(b_new, 0)
        assert np.array_equal(y2[inside], y[inside])
    if b_new == b_old:
        assert np.array_equal(got, c) and np.array_equal(oracle.repack(u, 0, b_old, b_new), u)


def test_repack_keeps_block_maximum_at_the_scale(oracle):
    for b_old in BITS:
        for b_new in BITS:
            qo, qn = 2 ** (b_old - 1) - 1, 2 ** (b_new - 1) - 1
            top = oracle.repack(np.array([0, qo, 2 * qo], np.uint8), 0, b_old, b_new)
            assert list(top) == [0, qn, 2 * qn]  # -s, 0, +s stay -s, 0, +s
            assert oracle.repack(np.array([2 ** b_old - 1], np.uint8), 1, b_old, b_new)[0] == 2 ** b_new - 1


def test_repack_log_narrowing_ties_take_larger_value(oracle):
    # 5 -> 4 bits: old level k=1 (2^-1/2) sits exactly on the new threshold between 1 and 2^-1
    c = np.array([31 - 1, 31 - 3], np.uint8)
    got = oracle.repack(c, 1, 5, 4)
    assert list(got) == [15 - 0, 15 - 1]


# ------------------------------------------------------------------ decision
def make_stats(oracle, g):
    s = oracle.Stats()
    g = g.astype(np.float64)
    s.count = g.size
    s.g_sum, s.g_abs_sum, s.g_sq_sum = g.sum(), np.abs(g).sum(), (g * g).sum()
    return s


def test_temporal_factor_closed_form(oracle):
    # Eq. 7: S_0 = 2, S -> 1; visible through the score of a single average layer (alpha = 1)
    c = read_constants()
    g = np.random.default_rng(1).standard_normal(1000)
    for t, tau in [(0, 100.0), (100, 100.0), (50000, 100.0)]:
        ema = oracle.Ema(0, 0, 0)
        _, _, sc = oracle.decide(ema, [make_stats(oracle, g)] * 3, t, alpha=1.0, tau=tau, eps=0.0)
        S = 1 + 1 / math.cosh(t / tau)
        assert abs(sc[0] - (c["phi"] + math.log2(S))) < 1e-12
    assert abs((1 + 1 / math.cosh(0.0)) - 2) == 0


def test_average_layer_gets_the_8bit_anchor(oracle):
    # Sec. 3.4: Phi = 7.2 anchors the 8-bit reference; thresholds 6.8 / 12 / 24
    c = read_constants()
    g = np.random.default_rng(2).standard_normal(4096) * 1e-3
    ema = oracle.Ema(0, 0, 0)
    bm, bv, sc = oracle.decide(ema, [make_stats(oracle, g)] * 4, 10 ** 9, alpha=1.0, eps=0.0)
    assert np.allclose(sc, c["phi"]) and list(bm) == [8] * 4 and list(bv) == [8] * 4
    assert oracle.PAPER_THRESHOLDS == tuple(c["thresholds"]) and oracle.PAPER_BITS == tuple(int(x) for x in c["bits"])
    assert oracle.PAPER_PHI == c["phi"]


def test_score_terms_and_map(oracle):
    # two layers, alpha = 1, t huge (S = 1): score_l = Phi + log2(r_l/rbar) + log2(n_l/nbar) + log2(v_l/vbar)
    rng = np.random.default_rng(3)
    g1 = rng.standard_normal(5000) * 1e-3
    g2 = rng.standard_normal(5000) * 4e-3 * np.exp(rng.standard_normal(5000))
    stats = [make_stats(oracle, g1), make_stats(oracle, g2)]
    ema = oracle.Ema(0, 0, 0)
    bm, bv, sc = oracle.decide(ema, stats, 10 ** 9, alpha=1.0, eps=0.0)
    n = [np.sqrt(np.mean(g * g)) for g in (g1, g2)]
    r = [np.std(np.abs(g)) / np.mean(np.abs(g)) for g in (g1, g2)]  # Eq. 3: CV of |g|
    v = [np.mean(g * g) for g in (g1, g2)]
    for l in range(2):
        want = 7.2 + math.log2(r[l] / np.mean(r)) + math.log2(n[l] / np.mean(n)) + math.log2(v[l] / np.mean(v))
        assert abs(sc[l] - want) < 1e-9
    assert abs(ema.n_ema - np.mean(n)) < 1e-15 and abs(ema.v_ema - np.mean(v)) < 1e-18
    # Alg. 1's variant of r_l uses sigma(g)
    ema = oracle.Ema(0, 0, 0)
    _, _, sc1 = oracle.decide(ema, stats, 10 ** 9, alpha=1.0, eps=0.0, r_mode=1)
    r1 = [np.std(g) / np.mean(np.abs(g)) for g in (g1, g2)]
    want = 7.2 + math.log2(r1[0] / np.mean(r1)) + math.log2(n[0] / np.mean(n)) + math.log2(v[0] / np.mean(v))
    assert abs(sc1[0] - want) < 1e-9


def test_ablations_drop_exactly_their_terms(oracle):
    # the component study's variants: each removes its own terms of the score and nothing else
    rng = np.random.default_rng(31)
    g1 = rng.standard_normal(4000) * 2e-3
    g2 = rng.standard_normal(4000) * 5e-4 * np.exp(0.5 * rng.standard_normal(4000))
    stats = [make_stats(oracle, g1), make_stats(oracle, g2)]
    t, tau = 30, 20.0
    full = oracle.decide(oracle.Ema(0, 0, 0), stats, t, alpha=1.0, tau=tau, eps=0.0)[2]
    n = [np.sqrt(np.mean(g * g)) for g in (g1, g2)]
    r = [np.std(np.abs(g)) / np.mean(np.abs(g)) for g in (g1, g2)]
    v = [np.mean(g * g) for g in (g1, g2)]
    dual = [math.log2(r[l] / np.mean(r)) + math.log2(n[l] / np.mean(n)) for l in range(2)]
    temporal = math.log2(1.0 + 1.0 / math.cosh(t / tau))
    spatial = [math.log2(v[l] / np.mean(v)) for l in range(2)]
    for drop, gone in ((1, dual), (2, [temporal] * 2), (4, spatial), (7, [dual[l] + temporal + spatial[l] for l in range(2)])):
        sc = oracle.decide(oracle.Ema(0, 0, 0), stats, t, alpha=1.0, tau=tau, eps=0.0, drop=drop)[2]
        for l in range(2):
            assert abs((full[l] - sc[l]) - gone[l]) < 1e-9, (drop, l)
    assert abs(oracle.decide(oracle.Ema(0, 0, 0), stats, t, alpha=1.0, tau=tau, eps=0.0, drop=7)[2][0] - 7.2) < 1e-12


def test_decision_cadence(oracle):
    # Algorithm 1: the decision runs when t mod U = 0 or t < 5
    due = [t for t in range(1, 41) if oracle.decide_due(t, 10)]
    assert due == [1, 2, 3, 4, 10, 20, 30, 40]
    assert [t for t in range(1, 12) if oracle.decide_due(t, 0)] == [1, 2, 3, 4]


def test_ema_recurrence_and_zero_init_bias(oracle):
    # Eq. 4 with EMAs initialised at 0 (Alg. 1): after one decision the EMA is alpha*mean, so every
    # ratio is 1/alpha and the score of an average layer is Phi + 3*log2(1/alpha) + log2(S)
    g = np.random.default_rng(4).standard_normal(2000)
    ema = oracle.Ema(0, 0, 0)
    st = [make_stats(oracle, g)] * 2
    _, _, sc = oracle.decide(ema, st, 10 ** 9, alpha=0.25, eps=0.0)
    assert abs(sc[0] - (7.2 + 3 * 2.0)) < 1e-9
    n0 = ema.n_ema
    oracle.decide(ema, st, 10 ** 9, alpha=0.25, eps=0.0)
    assert abs(ema.n_ema - (0.25 * (n0 / 0.25) + 0.75 * n0)) < 1e-15


def test_map_is_a_step_function_with_inclusive_thresholds(oracle):
    g = np.random.default_rng(5).standard_normal(1000)
    st = [make_stats(oracle, g)]
    for phi, want in [(6.79, 4), (6.8, 8), (11.99, 8), (12.0, 16), (23.9, 16), (24.0, 32), (100.0, 32), (-50.0, 4)]:
        ema = oracle.Ema(0, 0, 0)
        bm, _, sc = oracle.decide(ema, st, 10 ** 9, alpha=1.0, eps=0.0, phi=phi)
        assert sc[0] == phi and bm[0] == want
    # generic ladder and per-state offset
    ema = oracle.Ema(0, 0, 0)
    bm, bv, _ = oracle.decide(ema, st, 10 ** 9, alpha=1.0, eps=0.0, phi=5.0, v_offset=-1.0,
                              thr=(2.0, 3.0, 4.5, 5.0, 6.0), bits=(2, 3, 4, 5, 6, 8))
    assert bm[0] == 6 and bv[0] == 4
    # a layer with zero gradient scores -inf and takes the lowest width
    z = oracle.Stats()
    z.count = 10
    ema = oracle.Ema(0, 0, 0)
    bm, _, sc = oracle.decide(ema, [st[0], z], 5, alpha=0.5)
    assert sc[1] == -math.inf and bm[1] == 4
