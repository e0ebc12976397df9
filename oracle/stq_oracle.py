"""ctypes front end of the CPU oracle (stq_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It holds argument marshalling, and the outer iteration of
Algorithm 1 over steps and layers (`loop`: statistics as a by-product of the step,
decision applied one step later; `loop_alg1_order`: the order as written) as plain
Python control flow.  Every number comes out of the plain C in stq_oracle.c, which
is compiled here with gcc (fp32, no fused multiply-add, no fast-math).
Pins of the loops: tests/test_oracle_loop.py.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stq_oracle.c")
_LIB = os.path.join(_HERE, "libstq_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile stq_oracle.c into libstq_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class Stats(C.Structure):
    _fields_ = [
        ("count", C.c_uint64),
        ("g_sum", C.c_double), ("g_abs_sum", C.c_double), ("g_sq_sum", C.c_double), ("g_absmax", C.c_float),
        ("m_sum", C.c_double), ("m_sq_sum", C.c_double), ("m_err_sq", C.c_double), ("m_absmax", C.c_float),
        ("v_sum", C.c_double), ("v_sq_sum", C.c_double), ("v_err_sq", C.c_double), ("v_absmax", C.c_float),
    ]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class HParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_uint32)]


class Ema(C.Structure):
    _fields_ = [("n_ema", C.c_double), ("r_ema", C.c_double), ("v_ema", C.c_double)]


class DecideCfg(C.Structure):
    _fields_ = [("alpha", C.c_double), ("tau", C.c_double), ("phi", C.c_double), ("eps", C.c_double),
                ("v_offset", C.c_double), ("r_mode", C.c_int), ("n_thr", C.c_int),
                ("drop", C.c_int), ("pad_", C.c_int),
                ("thr", C.POINTER(C.c_double)), ("bits", C.POINTER(C.c_uint8))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.stq_oracle_G.restype = C.c_float
        L.stq_oracle_G.argtypes = [C.c_int]
        for f in (L.stq_oracle_R, L.stq_oracle_L, L.stq_oracle_T):
            f.restype = C.c_float
            f.argtypes = [C.c_int, C.c_int]
        L.stq_oracle_quant_linear_block.restype = C.c_float
        L.stq_oracle_quant_linear_block.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.stq_oracle_quant_log_block.restype = C.c_float
        L.stq_oracle_quant_log_block.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.stq_oracle_dequant_linear_block.restype = None
        L.stq_oracle_dequant_linear_block.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]
        L.stq_oracle_dequant_log_block.restype = None
        L.stq_oracle_dequant_log_block.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]
        L.stq_oracle_step.restype = None
        L.stq_oracle_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_uint64,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int, C.c_int, C.c_int, C.POINTER(HParams), C.POINTER(Stats)]
        L.stq_oracle_step_widths.restype = None
        L.stq_oracle_step_widths.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_uint64,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                             C.POINTER(HParams), C.POINTER(Stats)]
        L.stq_oracle_step_wide.restype = None
        L.stq_oracle_step_wide.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_uint64,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.POINTER(HParams), C.POINTER(Stats)]
        L.stq_oracle_wide_value.restype = C.c_float
        L.stq_oracle_wide_value.argtypes = [C.c_float, C.c_int]
        for f in (L.stq_oracle_pack_wide, L.stq_oracle_unpack_wide):
            f.restype = None
            f.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_void_p]
        L.stq_oracle_code_words.restype = C.c_uint64
        L.stq_oracle_code_words.argtypes = [C.c_uint64, C.c_int]
        L.stq_oracle_pack.restype = None
        L.stq_oracle_pack.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_void_p]
        L.stq_oracle_unpack.restype = None
        L.stq_oracle_unpack.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_void_p]
        L.stq_oracle_repack.restype = None
        L.stq_oracle_repack.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.stq_oracle_grad_stats.restype = None
        L.stq_oracle_grad_stats.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.POINTER(Stats)]
        L.stq_oracle_decide.restype = None
        L.stq_oracle_decide_due.restype = C.c_int
        L.stq_oracle_decide_due.argtypes = [C.c_uint32, C.c_uint32]
        L.stq_oracle_decide.argtypes = [C.POINTER(Ema), C.POINTER(Stats), C.c_int, C.POINTER(DecideCfg),
                                        C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    return a


# ---------------------------------------------------------------- tables
def G(j: int) -> np.float32:
    return np.float32(lib().stq_oracle_G(j))


def R(b: int, u: int) -> np.float32:
    return np.float32(lib().stq_oracle_R(b, u))


def Lv(b: int, c: int) -> np.float32:
    return np.float32(lib().stq_oracle_L(b, c))


def T(b: int, k: int) -> np.float32:
    return np.float32(lib().stq_oracle_T(b, k))


# ------------------------------------------------------------ quantizers
def quant_linear_block(x: np.ndarray, b: int):
    x = _chk(np.ascontiguousarray(x, dtype=np.float32), np.float32)
    u = np.empty(x.size, np.uint8)
    s = lib().stq_oracle_quant_linear_block(_p(x), x.size, b, _p(u))
    return u, np.float32(s)


def quant_log_block(x: np.ndarray, b: int):
    x = _chk(np.ascontiguousarray(x, dtype=np.float32), np.float32)
    c = np.empty(x.size, np.uint8)
    s = lib().stq_oracle_quant_log_block(_p(x), x.size, b, _p(c))
    return c, np.float32(s)


def dequant_linear_block(u: np.ndarray, b: int, s) -> np.ndarray:
    u = _chk(np.ascontiguousarray(u, dtype=np.uint8), np.uint8)
    x = np.empty(u.size, np.float32)
    lib().stq_oracle_dequant_linear_block(_p(u), u.size, b, C.c_float(float(s)), _p(x))
    return x


def dequant_log_block(c: np.ndarray, b: int, s) -> np.ndarray:
    c = _chk(np.ascontiguousarray(c, dtype=np.uint8), np.uint8)
    x = np.empty(c.size, np.float32)
    lib().stq_oracle_dequant_log_block(_p(c), c.size, b, C.c_float(float(s)), _p(x))
    return x


# ------------------------------------------------------------------ state
@dataclass
class State:
    """Unpacked optimizer state of one tensor: codes (one byte each) + block scales."""
    numel: int
    K: int
    bm: int
    bv: int
    um: np.ndarray = field(default=None)
    sm: np.ndarray = field(default=None)
    cv: np.ndarray = field(default=None)
    sv: np.ndarray = field(default=None)
    mw: np.ndarray = field(default=None)   # stored values of a first moment kept at 16 or 32 bits
    vw: np.ndarray = field(default=None)   # ... of a second moment

    @property
    def nblocks(self):
        return (self.numel + self.K - 1) // self.K

    @staticmethod
    def zeros(numel: int, K: int, bm: int, bv: int) -> "State":
        """Alg. 1 initial state m_0 = v_0 = 0: linear zero code is qmax, log blocks have scale 0."""
        nb = (numel + K - 1) // K
        qmax = (1 << (bm - 1)) - 1 if bm < 16 else 0
        return State(numel, K, bm, bv,
                     um=np.full(numel, qmax, np.uint8), sm=np.zeros(nb, np.float32),
                     cv=np.zeros(numel, np.uint8), sv=np.zeros(nb, np.float32),
                     mw=np.zeros(numel, np.float32) if bm >= 16 else None,
                     vw=np.zeros(numel, np.float32) if bv >= 16 else None)

    def copy(self):
        return State(self.numel, self.K, self.bm, self.bv, self.um.copy(), self.sm.copy(),
                     self.cv.copy(), self.sv.copy(),
                     None if self.mw is None else self.mw.copy(), None if self.vw is None else self.vw.copy())


def step(param: np.ndarray, grad: np.ndarray, st: State, *, lr, beta1, beta2, eps, weight_decay, t,
         want_stats: bool = False):
    """In-place Adam step of one tensor.  grad is float32, or uint16 holding bf16 bit patterns."""
    if st.bm >= 16 or st.bv >= 16:
        return step_transition(param, grad, st, st.bm, st.bv, lr=lr, beta1=beta1, beta2=beta2, eps=eps,
                               weight_decay=weight_decay, t=t, want_stats=want_stats)
    _chk(param, np.float32)
    assert param.size == st.numel and grad.size == st.numel
    bf16 = grad.dtype == np.uint16
    if not bf16:
        _chk(grad, np.float32)
    assert grad.flags.c_contiguous
    hp = HParams(lr, beta1, beta2, eps, weight_decay, t)
    stats = Stats() if want_stats else None
    lib().stq_oracle_step(_p(param), _p(grad), int(bf16), st.numel, _p(st.um), _p(st.sm), _p(st.cv), _p(st.sv),
                          st.bm, st.bv, st.K, C.byref(hp), C.byref(stats) if want_stats else None)
    return stats


def step_transition(param: np.ndarray, grad: np.ndarray, st: State, bm_new: int, bv_new: int, *, lr, beta1, beta2,
                    eps, weight_decay, t, want_stats: bool = False):
    """The step in which the layer's widths change (Algorithm 1: Map, then the layer loop): the stored
    moments are read at st.bm, st.bv and the new ones quantized at bm_new, bv_new.  Updates st in place,
    including its widths."""
    _chk(param, np.float32)
    assert param.size == st.numel and grad.size == st.numel
    bf16 = grad.dtype == np.uint16
    if not bf16:
        _chk(grad, np.float32)
    assert grad.flags.c_contiguous
    hp = HParams(lr, beta1, beta2, eps, weight_decay, t)
    stats = Stats() if want_stats else None
    if max(st.bm, bm_new) >= 16 and st.mw is None:
        st.mw = np.zeros(st.numel, np.float32)
    if max(st.bv, bv_new) >= 16 and st.vw is None:
        st.vw = np.zeros(st.numel, np.float32)
    lib().stq_oracle_step_wide(_p(param), _p(grad), int(bf16), st.numel, _p(st.um), _p(st.sm), _p(st.cv), _p(st.sv),
                               _p(st.mw) if st.mw is not None else None, _p(st.vw) if st.vw is not None else None,
                               st.bm, st.bv, bm_new, bv_new, st.K, C.byref(hp),
                               C.byref(stats) if want_stats else None)
    st.bm, st.bv = bm_new, bv_new
    return stats


# ----------------------------------------------------------------- layout
def code_words(numel: int, b: int) -> int:
    return int(lib().stq_oracle_code_words(numel, b))


def pack(codes: np.ndarray, b: int) -> np.ndarray:
    codes = _chk(np.ascontiguousarray(codes, dtype=np.uint8), np.uint8)
    w = np.empty(code_words(codes.size, b), np.uint32)
    lib().stq_oracle_pack(_p(codes), codes.size, b, _p(w))
    return w


def pack_wide(vals: np.ndarray, b: int) -> np.ndarray:
    """Storage words of a state kept at 16 or 32 bits."""
    vals = _chk(np.ascontiguousarray(vals, dtype=np.float32), np.float32)
    w = np.empty(code_words(vals.size, b), np.uint32)
    lib().stq_oracle_pack_wide(_p(vals), vals.size, b, _p(w))
    return w


def unpack_wide(words: np.ndarray, numel: int, b: int) -> np.ndarray:
    words = _chk(np.ascontiguousarray(words, dtype=np.uint32), np.uint32)
    assert words.size >= code_words(numel, b)
    v = np.empty(numel, np.float32)
    lib().stq_oracle_unpack_wide(_p(words), numel, b, _p(v))
    return v


def wide_value(x: float, b: int) -> float:
    return float(lib().stq_oracle_wide_value(float(np.float32(x)), b))


def unpack(words: np.ndarray, numel: int, b: int) -> np.ndarray:
    words = _chk(np.ascontiguousarray(words, dtype=np.uint32), np.uint32)
    assert words.size >= code_words(numel, b)
    c = np.empty(numel, np.uint8)
    lib().stq_oracle_unpack(_p(words), numel, b, _p(c))
    return c


def pad_scales(s: np.ndarray, numel: int, K: int) -> np.ndarray:
    """Scales as stored: zero-padded to 2048/K entries per 2048-element tile."""
    tiles = (numel + 2047) // 2048
    out = np.zeros(tiles * (2048 // K), np.float32)
    out[: s.size] = s
    return out


def repack(codes: np.ndarray, state: int, b_old: int, b_new: int) -> np.ndarray:
    codes = _chk(np.ascontiguousarray(codes, dtype=np.uint8), np.uint8)
    out = np.empty_like(codes)
    lib().stq_oracle_repack(_p(codes), codes.size, state, b_old, b_new, _p(out))
    return out


# --------------------------------------------------------------- decision
PAPER_THRESHOLDS = (6.8, 12.0, 24.0)
PAPER_BITS = (4, 8, 16, 32)
PAPER_PHI = 7.2


def decide_due(step_t: int, U: int) -> bool:
    return bool(lib().stq_oracle_decide_due(step_t, U))


def decide(ema: Ema, stats: list, step_t: int, *, alpha=0.1, tau=1000.0, phi=PAPER_PHI, eps=1e-12,
           v_offset=0.0, r_mode=0, thr=PAPER_THRESHOLDS, bits=PAPER_BITS, drop=0):
    L = len(stats)
    arr = (Stats * L)(*stats)
    thr_a = (C.c_double * len(thr))(*thr)
    bits_a = (C.c_uint8 * len(bits))(*bits)
    assert len(bits) == len(thr) + 1
    cfg = DecideCfg(alpha, tau, phi, eps, v_offset, r_mode, len(thr), drop, 0, thr_a, bits_a)
    bm = np.empty(L, np.uint8)
    bv = np.empty(L, np.uint8)
    sc = np.empty(L, np.float64)
    lib().stq_oracle_decide(C.byref(ema), arr, L, C.byref(cfg), step_t, _p(bm), _p(bv), _p(sc))
    return bm, bv, sc


def grad_stats(grad: np.ndarray) -> Stats:
    """Statistics of a layer's gradient alone (inputs of Eq. 2, 3, 8)."""
    bf16 = grad.dtype == np.uint16
    if not bf16:
        _chk(grad, np.float32)
    assert grad.flags.c_contiguous
    st = Stats()
    lib().stq_oracle_grad_stats(_p(grad), int(bf16), grad.size, C.byref(st))
    return st


def loop_alg1_order(params: list, states: list, grads_of_step, steps: int, U: int, hp: dict, decide_kw: dict,
                    ema: Ema = None, first_step: int = 1):
    """Algorithm 1 in the order it is written: at a decision step t the layer statistics of g_t go
    through the Score Engine and Map FIRST, and the layer loop of the same step t already quantizes at
    the new widths (reading the stored states at the old ones).  Returns (records (t, plan written in
    that step, scores or None), the EMAs)."""
    ema = ema if ema is not None else Ema(0.0, 0.0, 0.0)
    log = []
    for t in range(first_step, first_step + steps):
        grads = grads_of_step(t)
        plan, scores = [(st.bm, st.bv) for st in states], None
        if decide_due(t, U):
            bm, bv, scores = decide(ema, [grad_stats(g) for g in grads], t, **decide_kw)
            plan = [(int(a), int(b)) for a, b in zip(bm, bv)]
        for p, g, st, (bm, bv) in zip(params, grads, states, plan):
            step_transition(p, g, st, bm, bv, t=t, **hp)
        log.append((t, plan, scores))
    return log, ema


def loop(params: list, states: list, grads_of_step, steps: int, U: int, hp: dict, decide_kw: dict, ema: Ema = None,
         first_step: int = 1, next_plan: list = None):
    """Algorithm 1's iteration over a model of several layers, for steps first_step .. first_step+steps-1:
    every step runs the layer loop; when the cadence says so (t mod U = 0 or t < 5) the layer statistics
    of that step's gradients go through the Score Engine and Map.  The statistics are those gathered
    during the step, so the widths Map returns are the ones the NEXT step writes (it reads the states at
    the old widths).  params[l], states[l] are updated in place; grads_of_step(t) returns the list of
    gradient arrays of step t.  next_plan: the widths the first of these steps writes, when an earlier
    decision is still to take effect (default: the stored widths).  Returns (a list of per-step records
    (t, plan written in that step, scores or None), the widths the following step would write, the EMAs)."""
    ema = ema if ema is not None else Ema(0.0, 0.0, 0.0)
    nxt = list(next_plan) if next_plan is not None else [(st.bm, st.bv) for st in states]
    log = []
    for t in range(first_step, first_step + steps):
        due = decide_due(t, U)
        grads = grads_of_step(t)
        stats = []
        for p, g, st, (bm, bv) in zip(params, grads, states, nxt):
            stats.append(step_transition(p, g, st, bm, bv, t=t, want_stats=due, **hp))
        written, scores = list(nxt), None
        if due:
            bm, bv, scores = decide(ema, stats, t, **decide_kw)
            nxt = [(int(a), int(b)) for a, b in zip(bm, bv)]
        log.append((t, written, scores))
    return log, nxt, ema
