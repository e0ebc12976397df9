"""CPU-side checks of the C-ABI library: it loads, exports what include/stq.h declares, and its
host-only entry points (sizes, tables, decision, argument checks) behave.  No kernel is launched."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import paper_2604_06836_amd as stq
from paper_2604_06836_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BITS = [2, 3, 4, 5, 6, 7, 8]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(stq.library_path()):
        from paper_2604_06836_amd.build import build
        build()
    return stq.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "stq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(stq_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_state_bytes(lib):
    # one tile = 2048 elements = 64*b words of codes and 2048/K scales
    assert stq.state_bytes(1, 128, 4) == (64 * 4 * 4, 16 * 4)
    assert stq.state_bytes(2048, 64, 8) == (64 * 8 * 4, 32 * 4)
    assert stq.state_bytes(2049, 256, 3) == (2 * 64 * 3 * 4, 2 * 8 * 4)
    n = 768 * 3072
    cb, sb = stq.state_bytes(n, 128, 5)
    assert cb == n * 5 // 8 and sb == n // 128 * 4
    with pytest.raises(stq.StqError) as e:
        stq.state_bytes(10, 100, 4)
    assert e.value.code == -4
    with pytest.raises(stq.StqError) as e:
        stq.state_bytes(10, 128, 9)
    assert e.value.code == -3
    with pytest.raises(stq.StqError) as e:
        stq.state_bytes(0, 128, 4)
    assert e.value.code == -1


def test_scale_bytes_match_the_hand_cases(lib):
    # the library's scale-array size against the hand-derived cases that also pin the oracle's padding
    n_cases = 0
    for line in open(os.path.join(ROOT, "tests", "golden", "scale_padding_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        lhs, rhs = line.split("->")
        numel, K = (int(t) for t in lhs.split())
        _, stored = (int(t) for t in rhs.split())
        assert stq.state_bytes(numel, K, 4)[1] == 4 * stored, line
        n_cases += 1
    assert n_cases == 7


def test_tables_are_bit_identical_to_the_oracles(lib, oracle):
    # the library and the oracle build their tables independently; the codes can only agree
    # bit for bit if the tables do
    g = np.array(stq.table(0), np.float32)
    assert g.size == 511
    assert np.array_equal(g.view(np.uint32), np.array([oracle.G(j) for j in range(511)], np.float32).view(np.uint32))
    for b in BITS:
        r = np.array(stq.table(1, b), np.float32)
        l = np.array(stq.table(2, b), np.float32)
        t = np.array(stq.table(3, b), np.float32)
        assert r.size == 2 ** b - 1 and l.size == 2 ** b and t.size == 2 ** b - 1
        assert np.array_equal(r.view(np.uint32), np.array([oracle.R(b, u) for u in range(r.size)], np.float32).view(np.uint32))
        assert np.array_equal(l.view(np.uint32), np.array([oracle.Lv(b, c) for c in range(l.size)], np.float32).view(np.uint32))
        assert np.array_equal(t.view(np.uint32), np.array([oracle.T(b, k) for k in range(t.size)], np.float32).view(np.uint32))


def test_strerror(lib):
    assert stq.strerror(0) == "ok"
    assert "gfx950" in stq.strerror(-5)
    assert stq.strerror(-12345) == "unknown error"


def test_init_without_gpu_reports_device_error(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = C.c_void_p()
    assert lib.stq_init(C.byref(h), 0, 16) == -5
    assert lib.stq_init(None, 0, 16) == -1
    assert lib.stq_init(C.byref(h), 0, 0) == -1


def _stats_from(g):
    s = binding.LayerStats()
    g = np.asarray(g, np.float64)
    s.count = g.size
    s.g_sum, s.g_abs_sum, s.g_sq_sum = g.sum(), np.abs(g).sum(), (g * g).sum()
    return s


def test_decide_matches_oracle(lib, oracle):
    rng = np.random.default_rng(17)
    L = 40
    ladder = dict(thr=(4.0, 5.5, 7.0, 8.5, 10.0), bits=(2, 3, 4, 5, 6, 8))
    e_lib, e_or = binding.DecideState(0, 0, 0), oracle.Ema(0, 0, 0)
    for step in (1, 2, 3, 50, 1000):
        gs = [rng.standard_normal(int(rng.integers(100, 5000))) * 10 ** rng.uniform(-5, -2) for _ in range(L)]
        st_lib = [_stats_from(g) for g in gs]
        st_or = []
        for g in gs:
            s = oracle.Stats()
            s.count, s.g_sum, s.g_abs_sum, s.g_sq_sum = g.size, g.sum(), np.abs(g).sum(), (g * g).sum()
            st_or.append(s)
        for flags in (0, stq.STQ_DECIDE_R_ALG1, binding.STQ_DECIDE_NO_DUAL, binding.STQ_DECIDE_NO_TEMPORAL,
                      binding.STQ_DECIDE_NO_SPATIAL | stq.STQ_DECIDE_R_ALG1, 14):
            a, b = binding.DecideState(e_lib.n_ema, e_lib.r_ema, e_lib.v_ema), oracle.Ema(e_or.n_ema, e_or.r_ema, e_or.v_ema)
            plan, sc = stq.decide(a, st_lib, step, alpha=0.3, tau=40.0, v_offset=-1.0, flags=flags, **ladder)
            bm, bv, sc_o = oracle.decide(b, st_or, step, alpha=0.3, tau=40.0, v_offset=-1.0, r_mode=flags & 1,
                                         drop=flags >> 1, **ladder)
            np.testing.assert_allclose(sc, sc_o, rtol=0, atol=1e-9)
            thr = np.array(ladder["thr"])
            for l in range(L):
                near = np.min(np.abs(thr - sc_o[l])) < 1e-6 or np.min(np.abs(thr - (sc_o[l] - 1.0))) < 1e-6
                if not near:
                    assert plan[l] == (bm[l], bv[l])
        stq.decide(e_lib, st_lib, step, alpha=0.3, tau=40.0, **ladder)
        oracle.decide(e_or, st_or, step, alpha=0.3, tau=40.0, **ladder)
        assert abs(e_lib.n_ema - e_or.n_ema) <= 1e-15 * abs(e_or.n_ema)
        assert abs(e_lib.r_ema - e_or.r_ema) <= 1e-15 * abs(e_or.r_ema)
        assert abs(e_lib.v_ema - e_or.v_ema) <= 1e-15 * abs(e_or.v_ema)


def test_decide_due_matches_oracle(lib, oracle):
    for U in (0, 1, 7, 50):
        for t in range(1, 120):
            assert binding.decide_due(t, U) == oracle.decide_due(t, U)


def test_decide_paper_defaults(lib):
    # an exactly average layer, late in training (S = 1), alpha = 1: score = Phi = 7.2 -> 8 bits
    g = np.random.default_rng(3).standard_normal(1000)
    plan, sc = stq.decide(binding.DecideState(0, 0, 0), [_stats_from(g)] * 3, 10 ** 6, alpha=1.0, eps=0.0)
    assert all(abs(s - 7.2) < 1e-12 for s in sc) and plan == [(8, 8)] * 3
    # at t = 0 the temporal factor is 2: +1 bit of score
    plan, sc = stq.decide(binding.DecideState(0, 0, 0), [_stats_from(g)] * 3, 0, alpha=1.0, eps=0.0)
    assert all(abs(s - 8.2) < 1e-12 for s in sc)


def test_decide_argument_checks(lib):
    st = (binding.LayerStats * 1)(_stats_from([1.0, 2.0]))
    plan = (binding.Bits * 1)()
    thr = (C.c_double * 1)(5.0)
    bits = (C.c_uint8 * 2)(4, 8)
    cfg = binding.DecideCfg(0.1, 100.0, 7.2, 1e-12, 0.0, 0, 1, thr, bits)
    ema = binding.DecideState(0, 0, 0)
    assert lib.stq_decide(C.byref(ema), st, 1, C.byref(cfg), 1, plan, None) == 0
    assert lib.stq_decide(None, st, 1, C.byref(cfg), 1, plan, None) == -1
    assert lib.stq_decide(C.byref(ema), st, 0, C.byref(cfg), 1, plan, None) == -1
    bad = binding.DecideCfg(0.1, 0.0, 7.2, 1e-12, 0.0, 0, 1, thr, bits)  # tau must be positive
    assert lib.stq_decide(C.byref(ema), st, 1, C.byref(bad), 1, plan, None) == -1
    empty = (binding.LayerStats * 1)()
    assert lib.stq_decide(C.byref(ema), empty, 1, C.byref(cfg), 1, plan, None) == -1  # count == 0


def test_engine_entry_points_reject_null_handles(lib):
    # no device is touched before the handles are checked
    hp = binding.HParams(1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 128, 0, 0)
    out = C.c_void_p()
    assert lib.stq_engine_create(None, C.byref(out), None, None, 1, None, 8, 128, None, None, 0, None) == -1
    assert not out.value
    assert lib.stq_engine_create(None, None, None, None, 1, None, 8, 128, None, None, 0, None) == -1
    assert lib.stq_engine_step(None, C.byref(hp), 10, None, None) == -1
    assert lib.stq_engine_read(None, None, None, None, None, None, None) == -1
    assert lib.stq_engine_destroy(None) == -1


def test_header_is_plain_c():
    # the boundary is a C ABI: the header must compile as C99 on its own
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "stq.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
