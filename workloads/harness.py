"""Device-memory plumbing around the C-ABI library for tests and bench.py: allocates the
parameter, gradient and packed-state buffers of a workload as torch tensors and hands their
addresses to the binding.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np
import torch

import paper_2604_06836_amd as stq
from paper_2604_06836_amd import binding

from .configs import Workload


def hparams(w: Workload, t: int, stats=False) -> binding.HParams:
    """stats: False, True (every statistic) or "grad" (the gradient's only)."""
    h = w.hparams
    flags = stq.STQ_FLAG_STATS_GRAD if stats == "grad" else (stq.STQ_FLAG_STATS if stats else 0)
    return binding.HParams(h["lr"], h["beta1"], h["beta2"], h["eps"], h["weight_decay"], t, w.K,
                           1 if w.grad_dtype == "bf16" else 0, flags)


class DeviceModel:
    """All tensors of one workload resident on one GPU."""

    def __init__(self, ctx: stq.Context, w: Workload, plan: Sequence[Tuple[int, int]], device="cuda:0",
                 init_params: bool = True, spare_width: int = 0):
        """spare_width > 0: every state gets two code buffers of that width up front (the one in use is a
        view of the first), so that later width changes allocate nothing."""
        self.ctx, self.w, self.device = ctx, w, torch.device(device)
        self.plan = [tuple(p) for p in plan]
        self.param: List[torch.Tensor] = []
        self.grad: List[torch.Tensor] = []
        self.m_codes: List[torch.Tensor] = []
        self.v_codes: List[torch.Tensor] = []
        self.m_scales: List[torch.Tensor] = []
        self.v_scales: List[torch.Tensor] = []
        self._spare, self._cw = {}, {}     # (tensor, state) -> spare code buffer; cache of code sizes
        self._whole = None                 # address tables of the all-at-once path of apply_plan (spare_width only)
        self.repack_bytes = 0              # code bytes read and written by the re-pack launches so far
        self._spare_width = spare_width
        self.numel = [n for _, n in w.tensors]
        gdt = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
        for l, (_, n) in enumerate(w.tensors):
            bm, bv = self.plan[l]
            self.param.append(w.gen_param(l, self.device) if init_params
                              else torch.zeros(n, dtype=torch.float32, device=self.device))
            self.grad.append(torch.zeros(n, dtype=gdt, device=self.device))
            cb_m, sb = stq.state_bytes(n, w.K, bm)
            cb_v, _ = stq.state_bytes(n, w.K, bv)
            if spare_width:
                cb_max, _ = stq.state_bytes(n, w.K, spare_width)
                for state, lst in ((0, self.m_codes), (1, self.v_codes)):
                    lst.append(torch.empty(cb_max // 4, dtype=torch.int32, device=self.device))
                    self._spare[(l, state)] = torch.empty(cb_max // 4, dtype=torch.int32, device=self.device)
            else:
                self.m_codes.append(torch.empty(cb_m // 4, dtype=torch.int32, device=self.device))
                self.v_codes.append(torch.empty(cb_v // 4, dtype=torch.int32, device=self.device))
            self.m_scales.append(torch.empty(sb // 4, dtype=torch.float32, device=self.device))
            self.v_scales.append(torch.empty(sb // 4, dtype=torch.float32, device=self.device))
        self._rebuild()
        self.ctx.zero_state(self.tensors, self.cplan, w.K, self.stream)
        torch.cuda.synchronize(self.device)

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def _rebuild(self):
        self.tensors = binding.make_tensors(
            dict(param=p.data_ptr(), grad=g.data_ptr(), numel=p.numel(), m_codes=mc.data_ptr(),
                 m_scales=ms.data_ptr(), v_codes=vc.data_ptr(), v_scales=vs.data_ptr())
            for p, g, mc, ms, vc, vs in zip(self.param, self.grad, self.m_codes, self.m_scales,
                                            self.v_codes, self.v_scales))
        self.cplan = binding.make_plan(self.plan)

    def set_grads(self, step: int):
        for l in range(len(self.param)):
            self.grad[l].copy_(self.w.gen_grad(l, step, self.device))

    def step(self, t: int, stats=False):
        self.ctx.step(self.tensors, self.cplan, hparams(self.w, t, stats), self.stream)

    def _code_words(self, n: int, b: int) -> int:
        key = (n, b)
        if key not in self._cw:
            self._cw[key] = stq.state_bytes(n, self.w.K, b)[0] // 4
        return self._cw[key]

    def _destinations(self, new_plan):
        """For every state whose width changes: a destination buffer (the state's spare, or a new one
        sized for the widest quantized code).  Code buffers may be larger than the state needs."""
        out = []
        for l, ((bm0, bv0), (bm1, bv1)) in enumerate(zip(self.plan, new_plan)):
            if bm0 == bm1 and bv0 == bv1:
                continue
            n = self.numel[l]
            for state, cur, b0, b1 in ((0, self.m_codes, bm0, bm1), (1, self.v_codes, bv0, bv1)):
                if b0 == b1:
                    continue
                need = self._code_words(n, b1)
                spare = self._spare.get((l, state))
                if spare is None or spare.numel() < need:
                    spare = torch.empty(self._code_words(n, max(8, b1)), dtype=torch.int32, device=self.device)
                out.append((l, state, cur, b0, b1, spare, spare.data_ptr()))
        return out

    def _adopt(self, changes, new_plan, new_cplan, also_patch):
        self._whole = None
        arrays = (self.tensors,) + tuple(also_patch)
        for l, state, cur, b0, b1, dst, ptr in changes:
            self._spare[(l, state)] = cur[l]
            cur[l] = dst
            for arr in arrays:
                if state == 0:
                    arr[l].m_codes = ptr
                else:
                    arr[l].v_codes = ptr
        self.plan = [tuple(p) for p in new_plan]
        self.cplan = new_cplan

    def apply_plan(self, new_plan: Sequence[Tuple[int, int]], batched: bool = True, also_patch=()) -> int:
        """Re-pack every state whose width changed (out of place) and adopt the new plan.
        Returns the number of re-packed states.  Destination buffers come from a per-state spare
        (the buffer the state used before) so that a loop of transitions allocates nothing once warm.
        `also_patch`: further ctypes tensor arrays (other gradient sets of the same model) whose
        code pointers follow."""
        if batched and self._spare_width and max(max(p) for p in new_plan) <= self._spare_width:
            return self._apply_plan_whole(new_plan, also_patch)
        self._whole = None
        changes = self._destinations(new_plan)
        jobs = [(self.numel[l], state, cur[l].data_ptr(), b0, ptr, b1) for l, state, cur, b0, b1, dst, ptr in changes]
        self.repack_bytes += sum(((n + 2047) // 2048) * 256 * (b0 + b1) for n, _, _, b0, _, b1 in jobs)
        if batched and jobs:
            self.ctx.repack_many(jobs, self.w.K, self.stream)
        else:
            for n, state, src, b0, dst, b1 in jobs:
                self.ctx.repack(n, self.w.K, state, src, b0, dst, b1, self.stream)
        self._adopt(changes, new_plan, binding.make_plan(new_plan), also_patch)
        return len(changes)

    def _apply_plan_whole(self, new_plan, also_patch) -> int:
        """apply_plan when every state has both of its buffers at full capacity (spare_width): the job table
        and the patched tensor arrays are built with array operations instead of a Python loop per change."""
        if self._whole is None:
            L = len(self.numel)
            self._whole = dict(
                cur=[np.array([t.data_ptr() for t in lst], np.uint64) for lst in (self.m_codes, self.v_codes)],
                spare=[np.array([self._spare[(l, st)].data_ptr() for l in range(L)], np.uint64) for st in (0, 1)],
                numel=np.array(self.numel, np.uint64), plan=np.array(self.plan, np.uint8))
        wh = self._whole
        new = np.asarray(new_plan, np.uint8)
        idx = [np.nonzero(wh["plan"][:, st] != new[:, st])[0] for st in (0, 1)]
        jobs = np.zeros(len(idx[0]) + len(idx[1]), binding.REPACK_JOB_DTYPE)
        at = 0
        for st in (0, 1):
            j = jobs[at:at + len(idx[st])]
            j["numel"], j["src_codes"], j["dst_codes"] = wh["numel"][idx[st]], wh["cur"][st][idx[st]], wh["spare"][st][idx[st]]
            j["state"], j["src_bits"], j["dst_bits"] = st, wh["plan"][idx[st], st], new[idx[st], st]
            at += len(idx[st])
        if len(jobs):
            self.ctx.repack_many(jobs, self.w.K, self.stream)
            tiles = (jobs["numel"] + np.uint64(2047)) // np.uint64(2048)
            self.repack_bytes += int((tiles * 256 * (jobs["src_bits"].astype(np.uint64) + jobs["dst_bits"])).sum())
        views = [np.frombuffer(arr, dtype=binding.TENSOR_DTYPE) for arr in (self.tensors,) + tuple(also_patch)]
        for st, (lst, field) in enumerate(((self.m_codes, "m_codes"), (self.v_codes, "v_codes"))):
            i = idx[st]
            wh["cur"][st][i], wh["spare"][st][i] = wh["spare"][st][i], wh["cur"][st][i].copy()
            for v in views:
                v[field][i] = wh["cur"][st][i]
            for l in i.tolist():   # the tensor objects follow their addresses
                lst[l], self._spare[(l, st)] = self._spare[(l, st)], lst[l]
        wh["plan"] = new.copy()
        self.plan = [tuple(p) for p in new.tolist()]
        self.cplan = (binding.Bits * len(self.plan))()
        np.frombuffer(self.cplan, dtype=binding.BITS_DTYPE)["m_bits"][:] = new[:, 0]
        np.frombuffer(self.cplan, dtype=binding.BITS_DTYPE)["v_bits"][:] = new[:, 1]
        return len(jobs)

    def step_transition(self, t: int, new_plan: Sequence[Tuple[int, int]], stats=False, also_patch=()) -> int:
        """One step that reads the states at the current plan and writes them at new_plan
        (stq_step_transition), then adopts the new buffers and plan.  Returns the number of changed states."""
        changes = self._destinations(new_plan)
        dests = [[None, None] for _ in self.plan]
        for l, state, cur, b0, b1, dst, ptr in changes:
            dests[l][state] = ptr
        new_cplan = binding.make_plan(new_plan)
        self.ctx.step_transition(self.tensors, self.cplan, new_cplan, dests, hparams(self.w, t, stats), self.stream)
        self._adopt(changes, new_plan, new_cplan, also_patch)
        return len(changes)

    # ----------------------------------------------------------- host copies
    def host_state(self, l: int):
        """(param, m_code_words, m_scales, v_code_words, v_scales) of tensor l as numpy arrays."""
        bm, bv = self.plan[l]
        nm, nv = self._code_words(self.numel[l], bm), self._code_words(self.numel[l], bv)
        return (self.param[l].cpu().numpy(),
                self.m_codes[l][:nm].cpu().numpy().view(np.uint32), self.m_scales[l].cpu().numpy(),
                self.v_codes[l][:nv].cpu().numpy().view(np.uint32), self.v_scales[l].cpu().numpy())

    def host_grad(self, l: int) -> np.ndarray:
        g = self.grad[l]
        if g.dtype == torch.bfloat16:
            return g.view(torch.int16).cpu().numpy().view(np.uint16)
        return g.cpu().numpy()
