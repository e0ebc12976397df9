"""ctypes binding of include/stq.h.  Same names as the C entry points, argument marshalling only.

Device buffers are passed as integer addresses (e.g. torch.Tensor.data_ptr()); streams as the
integer hipStream_t (torch.cuda.current_stream().cuda_stream).  There is no fallback: if
libstq.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Iterable, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("STQ_LIBRARY", os.path.join(_PKG, "libstq.so"))  # override: another build of the same ABI

STQ_FLAG_STATS = 1
STQ_FLAG_STATS_GRAD = 2
STQ_DECIDE_R_ALG1 = 1
STQ_DECIDE_NO_DUAL, STQ_DECIDE_NO_TEMPORAL, STQ_DECIDE_NO_SPATIAL = 2, 4, 8
STQ_ENGINE_ALG1_ORDER = 1


class StqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, strerror(code)))


class Tensor(C.Structure):
    _fields_ = [("param", C.c_void_p), ("grad", C.c_void_p), ("numel", C.c_uint64),
                ("m_codes", C.c_void_p), ("m_scales", C.c_void_p),
                ("v_codes", C.c_void_p), ("v_scales", C.c_void_p)]


class Bits(C.Structure):
    _fields_ = [("m_bits", C.c_uint8), ("v_bits", C.c_uint8)]


class HParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_uint32), ("block", C.c_uint32),
                ("grad_dtype", C.c_uint32), ("flags", C.c_uint32)]


class LayerStats(C.Structure):
    _fields_ = [
        ("count", C.c_uint64),
        ("g_sum", C.c_double), ("g_abs_sum", C.c_double), ("g_sq_sum", C.c_double), ("g_absmax", C.c_float),
        ("m_sum", C.c_double), ("m_sq_sum", C.c_double), ("m_err_sq", C.c_double), ("m_absmax", C.c_float),
        ("v_sum", C.c_double), ("v_sq_sum", C.c_double), ("v_err_sq", C.c_double), ("v_absmax", C.c_float),
    ]


class DecideState(C.Structure):
    _fields_ = [("n_ema", C.c_double), ("r_ema", C.c_double), ("v_ema", C.c_double)]


class DecideCfg(C.Structure):
    _fields_ = [("alpha", C.c_double), ("tau", C.c_double), ("phi", C.c_double), ("eps", C.c_double),
                ("v_offset", C.c_double), ("flags", C.c_uint32), ("n_thr", C.c_uint32),
                ("thr", C.POINTER(C.c_double)), ("bits", C.POINTER(C.c_uint8))]


class RepackJob(C.Structure):
    _fields_ = [("numel", C.c_uint64), ("src_codes", C.c_void_p), ("dst_codes", C.c_void_p),
                ("state", C.c_uint8), ("src_bits", C.c_uint8), ("dst_bits", C.c_uint8)]


# the same records as numpy dtypes, for callers that build or patch whole arrays at once
REPACK_JOB_DTYPE = np.dtype([("numel", "<u8"), ("src_codes", "<u8"), ("dst_codes", "<u8"),
                             ("state", "u1"), ("src_bits", "u1"), ("dst_bits", "u1")], align=True)
TENSOR_DTYPE = np.dtype([("param", "<u8"), ("grad", "<u8"), ("numel", "<u8"), ("m_codes", "<u8"), ("m_scales", "<u8"),
                         ("v_codes", "<u8"), ("v_scales", "<u8")])
BITS_DTYPE = np.dtype([("m_bits", "u1"), ("v_bits", "u1")])


class Codes(C.Structure):
    _fields_ = [("m_codes", C.c_void_p), ("v_codes", C.c_void_p)]


EXPORTS = ["stq_init", "stq_set_schedule", "stq_destroy", "stq_state_bytes", "stq_zero_state", "stq_step", "stq_step_static", "stq_step_transition", "stq_grad_stats", "stq_stats",
           "stq_repack", "stq_repack_many", "stq_decide", "stq_decide_due", "stq_engine_create", "stq_engine_set_next", "stq_engine_step",
           "stq_engine_read", "stq_engine_destroy", "stq_table", "stq_strerror"]

_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libstq.so.  Raises if it has not been built (python -m paper_2604_06836_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError("%s not found: build it with `python -m paper_2604_06836_amd.build`" % _LIB_PATH)
    L = C.CDLL(_LIB_PATH)
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    L.stq_init.argtypes = [C.POINTER(vp), C.c_int, u32]
    L.stq_set_schedule.argtypes = [vp, u64]
    L.stq_destroy.argtypes = [vp]
    L.stq_state_bytes.argtypes = [u64, u32, u32, C.POINTER(u64), C.POINTER(u64)]
    L.stq_zero_state.argtypes = [vp, C.POINTER(Tensor), u32, C.POINTER(Bits), u32, vp]
    L.stq_step.argtypes = [vp, C.POINTER(Tensor), u32, C.POINTER(Bits), C.POINTER(HParams), vp]
    L.stq_step_static.argtypes = L.stq_step.argtypes
    L.stq_step_transition.argtypes = [vp, C.POINTER(Tensor), u32, C.POINTER(Bits), C.POINTER(Bits),
                                      C.POINTER(Codes), C.POINTER(HParams), vp]
    L.stq_grad_stats.argtypes = [vp, C.POINTER(Tensor), u32, u32, u32, vp]
    L.stq_stats.argtypes = [vp, C.POINTER(LayerStats), u32, vp]
    L.stq_repack.argtypes = [vp, u64, u32, C.c_int, vp, u32, vp, u32, vp]
    L.stq_repack_many.argtypes = [vp, C.POINTER(RepackJob), u32, u32, vp]
    L.stq_decide.argtypes = [C.POINTER(DecideState), C.POINTER(LayerStats), u32, C.POINTER(DecideCfg), u32,
                             C.POINTER(Bits), C.POINTER(C.c_double)]
    L.stq_decide_due.argtypes = [u32, u32]
    L.stq_table.argtypes = [C.c_int, u32, C.POINTER(C.c_float), u32]
    L.stq_engine_create.argtypes = [vp, C.POINTER(vp), C.POINTER(Tensor), C.POINTER(Codes), u32, C.POINTER(Bits), u32,
                                    u32, C.POINTER(DecideCfg), C.POINTER(DecideState), u32, vp]
    L.stq_engine_set_next.argtypes = [vp, C.POINTER(Bits), vp]
    L.stq_engine_step.argtypes = [vp, C.POINTER(HParams), u32, C.POINTER(vp), vp]
    L.stq_engine_read.argtypes = [vp, C.POINTER(Bits), C.POINTER(Bits), C.POINTER(Codes), C.POINTER(C.c_double),
                                  C.POINTER(DecideState), vp]
    L.stq_engine_destroy.argtypes = [vp]
    for name in EXPORTS[:-1]:
        getattr(L, name).restype = C.c_int
    L.stq_strerror.argtypes = [C.c_int]
    L.stq_strerror.restype = C.c_char_p
    _lib = L
    return L


def strerror(code: int) -> str:
    try:
        return load_library().stq_strerror(code).decode()
    except Exception:  # library missing: still give the number a name
        return "error %d" % code


def _check(code: int, where: str):
    if code != 0:
        raise StqError(code, where)


def state_bytes(numel: int, block: int, bits: int):
    """(code_bytes, scale_bytes) of one state of a tensor."""
    cb, sb = C.c_uint64(), C.c_uint64()
    _check(load_library().stq_state_bytes(numel, block, bits, C.byref(cb), C.byref(sb)), "stq_state_bytes")
    return cb.value, sb.value


def table(which: int, bits: int = 0):
    """The library's quantizer tables (0: G, 1: R_b, 2: L_b, 3: T_b) as a list of floats."""
    buf = (C.c_float * 512)()
    n = load_library().stq_table(which, bits, buf, 512)
    if n < 0:
        raise StqError(n, "stq_table")
    return list(buf[:n])


def make_tensors(items: Iterable[dict]):
    """items: dicts with param, grad, numel, m_codes, m_scales, v_codes, v_scales (addresses or None)."""
    items = list(items)
    arr = (Tensor * len(items))()
    for a, it in zip(arr, items):
        a.param, a.grad, a.numel = it.get("param"), it.get("grad"), it["numel"]
        a.m_codes, a.m_scales = it["m_codes"], it["m_scales"]
        a.v_codes, a.v_scales = it["v_codes"], it["v_scales"]
    return arr


def make_plan(plan: Sequence) -> "C.Array":
    arr = (Bits * len(plan))()
    for a, p in zip(arr, plan):
        a.m_bits, a.v_bits = int(p[0]), int(p[1])
    return arr


def decide_due(step: int, update_every: int) -> bool:
    return bool(load_library().stq_decide_due(step, update_every))


def decide(ema: DecideState, stats, step: int, *, alpha=0.1, tau=1000.0, phi=7.2, eps=1e-12, v_offset=0.0,
           flags=0, thr=(6.8, 12.0, 24.0), bits=(4, 8, 16, 32)):
    """stq_decide: returns (plan [(m_bits, v_bits)], scores).  stats: ctypes array or list of LayerStats."""
    n = len(stats)
    if not isinstance(stats, C.Array):
        stats = (LayerStats * n)(*stats)
    thr_a = (C.c_double * len(thr))(*thr)
    bits_a = (C.c_uint8 * len(bits))(*bits)
    if len(bits) != len(thr) + 1:
        raise ValueError("bits must have len(thr)+1 entries")
    cfg = DecideCfg(alpha, tau, phi, eps, v_offset, flags, len(thr), thr_a, bits_a)
    plan = (Bits * n)()
    scores = (C.c_double * n)()
    _check(load_library().stq_decide(C.byref(ema), stats, n, C.byref(cfg), step, plan, scores), "stq_decide")
    return [(p.m_bits, p.v_bits) for p in plan], list(scores)


class Context:
    """Owns an stq_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0, max_tensors: int = 1024):
        self._lib = load_library()
        self._h = C.c_void_p()
        _check(self._lib.stq_init(C.byref(self._h), device, max_tensors), "stq_init")

    def close(self):
        if self._h:
            self._lib.stq_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_schedule(self, ticket_min_tiles: int):
        _check(self._lib.stq_set_schedule(self._h, ticket_min_tiles), "stq_set_schedule")

    def zero_state(self, tensors, plan, block: int, stream: int = 0):
        _check(self._lib.stq_zero_state(self._h, tensors, len(tensors), plan, block, C.c_void_p(stream)),
               "stq_zero_state")

    def step(self, tensors, plan, hp: HParams, stream: int = 0):
        _check(self._lib.stq_step(self._h, tensors, len(tensors), plan, C.byref(hp), C.c_void_p(stream)),
               "stq_step")

    def step_static(self, tensors, plan, hp: HParams, stream: int = 0):
        _check(self._lib.stq_step_static(self._h, tensors, len(tensors), plan, C.byref(hp), C.c_void_p(stream)),
               "stq_step_static")

    def step_transition(self, tensors, plan_old, plan_new, new_codes, hp: HParams, stream: int = 0):
        """new_codes: sequence of (m_ptr or None, v_ptr or None), one per tensor."""
        arr = (Codes * len(tensors))()
        for a, (m, v) in zip(arr, new_codes):
            a.m_codes, a.v_codes = m, v
        _check(self._lib.stq_step_transition(self._h, tensors, len(tensors), plan_old, plan_new, arr,
                                             C.byref(hp), C.c_void_p(stream)), "stq_step_transition")

    def grad_stats(self, tensors, block: int, grad_dtype: int, stream: int = 0):
        _check(self._lib.stq_grad_stats(self._h, tensors, len(tensors), block, grad_dtype, C.c_void_p(stream)),
               "stq_grad_stats")

    def stats(self, n: int, stream: int = 0):
        out = (LayerStats * n)()
        _check(self._lib.stq_stats(self._h, out, n, C.c_void_p(stream)), "stq_stats")
        return out

    def repack_many(self, jobs, block: int, stream: int = 0):
        """jobs: sequence of (numel, state, src_ptr, src_bits, dst_ptr, dst_bits), or a numpy array of
        REPACK_JOB_DTYPE records (the C struct's layout), which is passed as it is."""
        if isinstance(jobs, np.ndarray):
            assert jobs.dtype == REPACK_JOB_DTYPE and jobs.flags["C_CONTIGUOUS"]
            arr = jobs.ctypes.data_as(C.POINTER(RepackJob))
        else:
            arr = (RepackJob * len(jobs))()
            for i, (numel, state, src, sb, dst, db) in enumerate(jobs):
                arr[i] = RepackJob(numel, src, dst, state, sb, db)
        _check(self._lib.stq_repack_many(self._h, arr, len(jobs), block, C.c_void_p(stream)), "stq_repack_many")

    def repack(self, numel: int, block: int, state: int, src: int, src_bits: int, dst: int, dst_bits: int,
               stream: int = 0):
        _check(self._lib.stq_repack(self._h, numel, block, state, C.c_void_p(src), src_bits,
                                    C.c_void_p(dst), dst_bits, C.c_void_p(stream)), "stq_repack")

    def engine(self, tensors, second, plan, capacity_bits: int, block: int, *, alpha=0.1, tau=1000.0, phi=7.2,
               eps=1e-12, v_offset=0.0, flags=0, thr=(6.8, 12.0, 24.0), bits=(4, 8, 16, 32),
               ema: Optional[DecideState] = None, alg1_order: bool = False, stream: int = 0) -> "Engine":
        """stq_engine_create.  second: sequence of (m_ptr, v_ptr), the second code buffer of each state."""
        return Engine(self, tensors, second, plan, capacity_bits, block, alpha=alpha, tau=tau, phi=phi, eps=eps,
                      v_offset=v_offset, flags=flags, thr=thr, bits=bits, ema=ema, alg1_order=alg1_order, stream=stream)


class Engine:
    """Owns an stq_engine: the device-resident precision loop.  Close it before its Context."""

    def __init__(self, ctx: Context, tensors, second, plan, capacity_bits: int, block: int, *, alpha, tau, phi, eps,
                 v_offset, flags, thr, bits, ema, alg1_order, stream):
        if len(bits) != len(thr) + 1:
            raise ValueError("bits must have len(thr)+1 entries")
        self._lib, self._ctx, self.n = ctx._lib, ctx, len(tensors)
        self._h = C.c_void_p()
        thr_a = (C.c_double * len(thr))(*thr)
        bits_a = (C.c_uint8 * len(bits))(*bits)
        cfg = DecideCfg(alpha, tau, phi, eps, v_offset, flags, len(thr), thr_a, bits_a)
        sec = (Codes * self.n)()
        for a, (m, v) in zip(sec, second):
            a.m_codes, a.v_codes = m, v
        _check(self._lib.stq_engine_create(ctx._h, C.byref(self._h), tensors, sec, self.n, plan, capacity_bits, block,
                                           C.byref(cfg), C.byref(ema) if ema is not None else None,
                                           STQ_ENGINE_ALG1_ORDER if alg1_order else 0, C.c_void_p(stream)),
               "stq_engine_create")

    def step(self, hp: HParams, update_every: int, grads: Optional[Sequence[int]] = None, stream: int = 0):
        """grads: None, or the addresses of the n gradient buffers to use from this step on (a ctypes
        array of c_void_p is passed through as it is)."""
        if grads is not None and not isinstance(grads, C.Array):
            grads = (C.c_void_p * self.n)(*grads)
        _check(self._lib.stq_engine_step(self._h, C.byref(hp), update_every, grads, C.c_void_p(stream)),
               "stq_engine_step")

    def set_next(self, next_plan, stream: int = 0):
        """stq_engine_set_next: next_plan is a sequence of (m_bits, v_bits) or a ctypes array of Bits."""
        if not isinstance(next_plan, C.Array):
            next_plan = make_plan(next_plan)
        _check(self._lib.stq_engine_set_next(self._h, next_plan, C.c_void_p(stream)), "stq_engine_set_next")

    def read(self, stream: int = 0):
        """stq_engine_read: dict with stored and next plans [(m_bits, v_bits)], current code buffers
        [(m_ptr, v_ptr)], scores and the EMAs (n_ema, r_ema, v_ema)."""
        stored, nxt, cur = (Bits * self.n)(), (Bits * self.n)(), (Codes * self.n)()
        score, ema = (C.c_double * self.n)(), DecideState(0, 0, 0)
        _check(self._lib.stq_engine_read(self._h, stored, nxt, cur, score, C.byref(ema), C.c_void_p(stream)),
               "stq_engine_read")
        return dict(stored=[(p.m_bits, p.v_bits) for p in stored], next=[(p.m_bits, p.v_bits) for p in nxt],
                    current=[(c.m_codes, c.v_codes) for c in cur], score=list(score),
                    ema=(ema.n_ema, ema.r_ema, ema.v_ema))

    def close(self):
        if self._h:
            self._lib.stq_engine_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
