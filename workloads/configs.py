"""The five benchmark configurations as seeded synthetic workloads.

The paper trains GPT-2 / ViT models on OpenWebText, COCO 2017, Wikitext-103 and MNLI; none of
those datasets or weights are used here.  What stands in for them: parameter sets with the
models' tensor shapes, parameters ~ N(0, 0.02^2), and gradients drawn per tensor and per step
from the distribution each configuration names.  Every draw is seeded by
(configuration, step, tensor index).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

ADAM = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)


def _seed(cfg: int, step: int, tensor: int, salt: int = 0) -> int:
    return 1_000_003 * cfg + 1009 * step + tensor + 7_919_000_000 * salt


def gpt2_shapes(d: int, layers: int, vocab: int, ctx: int = 1024) -> List[Tuple[str, int]]:
    t = [("wte", vocab * d), ("wpe", ctx * d)]
    for i in range(layers):
        t += [(f"h{i}.ln1.w", d), (f"h{i}.ln1.b", d), (f"h{i}.qkv", d * 3 * d), (f"h{i}.proj", d * d),
              (f"h{i}.ln2.w", d), (f"h{i}.ln2.b", d), (f"h{i}.fc", d * 4 * d), (f"h{i}.fc2", 4 * d * d)]
    t += [("ln_f.w", d), ("ln_f.b", d)]
    return t


def vit_b16_shapes() -> List[Tuple[str, int]]:
    d = 768
    t = [("patch_embed", 768 * 768)]
    for i in range(12):
        t += [(f"b{i}.qkv", d * 3 * d), (f"b{i}.proj", d * d), (f"b{i}.fc", d * 4 * d), (f"b{i}.fc2", 4 * d * d)]
    t += [("head", d * 1000)]
    return t


def llama7b_slice_shapes(total: int = 3_500_000_000) -> List[Tuple[str, int]]:
    """A contiguous slice of a d=4096, ffn=11008, vocab=32000 model, cut at `total` elements."""
    d, f, vocab = 4096, 11008, 32000
    t: List[Tuple[str, int]] = [("tok_embeddings", vocab * d)]
    for i in range(32):
        t += [(f"l{i}.attn_norm", d), (f"l{i}.wq", d * d), (f"l{i}.wk", d * d), (f"l{i}.wv", d * d),
              (f"l{i}.wo", d * d), (f"l{i}.ffn_norm", d), (f"l{i}.w_gate", d * f), (f"l{i}.w_up", d * f),
              (f"l{i}.w_down", f * d)]
    out, acc = [], 0
    for name, n in t:
        if acc + n >= total:
            out.append((name + "[slice]", total - acc))
            break
        out.append((name, n))
        acc += n
    return out


@dataclass
class Workload:
    cfg: int                      # index into benchmark configs (0-based)
    name: str
    tensors: List[Tuple[str, int]]
    K: int
    grad_dtype: str               # "fp32" or "bf16"
    steps: int
    grad_kind: str                # "normal", "normal_per_tensor", "student_t", "normal_per_tensor_step"
    bits_m: Tuple[int, ...] = (8,)
    bits_v: Tuple[int, ...] = (4,)
    p_m: Optional[Tuple[float, ...]] = None
    p_v: Optional[Tuple[float, ...]] = None
    transitions: str = "none"     # "none", "switch10pct_every5", "decide_every_step"
    hparams: dict = field(default_factory=lambda: dict(ADAM))

    @property
    def numel(self) -> int:
        return sum(n for _, n in self.tensors)

    # ------------------------------------------------------------- bit plan
    def initial_plan(self) -> List[Tuple[int, int]]:
        rng = np.random.default_rng(_seed(self.cfg, 0, 0, salt=1))
        L = len(self.tensors)
        bm = rng.choice(self.bits_m, size=L, p=self.p_m)
        bv = rng.choice(self.bits_v, size=L, p=self.p_v)
        return [(int(a), int(b)) for a, b in zip(bm, bv)]

    def switch_plan(self, plan: List[Tuple[int, int]], step: int) -> List[Tuple[int, int]]:
        """Configuration 3: every 5 steps 10 % of the tensors change one state's width."""
        if self.transitions != "switch10pct_every5" or step % 5 != 0:
            return plan
        rng = np.random.default_rng(_seed(self.cfg, step, 0, salt=2))
        L = len(plan)
        out = list(plan)
        for l in rng.choice(L, size=max(1, L // 10), replace=False):
            bm, bv = out[l]
            which = int(rng.integers(0, 2))
            cur = (bm, bv)[which]
            new = int(rng.choice([b for b in (4, 5, 6, 8) if b != cur]))
            out[l] = (new, bv) if which == 0 else (bm, new)
        return out

    def avg_bits(self, plan) -> float:
        tot = sum(n for _, n in self.tensors)
        return sum(n * (bm + bv) for (_, n), (bm, bv) in zip(self.tensors, plan)) / (2 * tot)

    def bytes_per_param(self, plan) -> float:
        """Algorithmic HBM bytes per parameter of one step: theta read+write, gradient read,
        codes read+write, block scales read+write."""
        g = 4 if self.grad_dtype == "fp32" else 2
        tot = sum(n for _, n in self.tensors)
        code = sum(n * 2 * (bm + bv) / 8 for (_, n), (bm, bv) in zip(self.tensors, plan)) / tot
        return 8 + g + code + 16 / self.K

    # ------------------------------------------------------------- values
    def grad_sigma(self, l: int, step: int) -> float:
        if self.grad_kind == "normal":
            return 1e-3
        if self.grad_kind == "student_t":
            return 1e-3
        s = step if self.grad_kind == "normal_per_tensor_step" else 0
        rng = np.random.default_rng(_seed(self.cfg, s, l, salt=3))
        return float(10.0 ** rng.uniform(-5, -2))

    def gen_param(self, l: int, device="cpu") -> torch.Tensor:
        n = self.tensors[l][1]
        gen = torch.Generator(device=device)
        gen.manual_seed(_seed(self.cfg, 0, l, salt=4))
        return torch.randn(n, generator=gen, device=device, dtype=torch.float32) * 0.02

    def gen_grad(self, l: int, step: int, device="cpu") -> torch.Tensor:
        """fp32 tensor, or bf16 tensor (round to nearest even from fp32) for bf16 workloads."""
        n = self.tensors[l][1]
        gen = torch.Generator(device=device)
        gen.manual_seed(_seed(self.cfg, step, l, salt=5))
        z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        if self.grad_kind == "student_t":  # nu = 3: z / sqrt(chi2_3 / 3)
            chi = torch.zeros_like(z)
            for _ in range(3):
                chi += torch.randn(n, generator=gen, device=device, dtype=torch.float32) ** 2
            z = z / torch.sqrt(chi / 3.0)
        g = z * self.grad_sigma(l, step)
        return g.to(torch.bfloat16) if self.grad_dtype == "bf16" else g


_P4568 = (0.45, 0.22, 0.21, 0.12)  # over {4,5,6,8}: mean 5.12

WORKLOADS = {
    "adam-1tensor": Workload(0, "adam-1tensor", [("w", 768 * 3072)], 128, "fp32", 10, "normal"),
    "gpt2-small": Workload(1, "gpt2-small", gpt2_shapes(768, 12, 50257), 128, "fp32", 20, "normal_per_tensor",
                           bits_m=(4, 5, 6, 8), bits_v=(4, 5, 6, 8), p_m=_P4568, p_v=_P4568),
    "vit-b16": Workload(2, "vit-b16", vit_b16_shapes(), 256, "fp32", 50, "student_t",
                        bits_m=(6,), bits_v=(4,), transitions="switch10pct_every5"),
    "gpt2-xl": Workload(3, "gpt2-xl", gpt2_shapes(1600, 48, 50257), 128, "bf16", 10, "normal_per_tensor_step",
                        bits_m=(2, 3, 4, 5, 6, 8), bits_v=(2, 3, 4, 5, 6, 8),
                        p_m=(0.05, 0.1, 0.3, 0.25, 0.2, 0.1), p_v=(0.05, 0.1, 0.3, 0.25, 0.2, 0.1),
                        transitions="decide_every_step"),
    "llama7b-slice": Workload(4, "llama7b-slice", llama7b_slice_shapes(), 64, "bf16", 5, "normal_per_tensor",
                              bits_m=(4, 5, 6, 7, 8), bits_v=(3, 4, 5, 6),
                              p_m=(0.3, 0.3, 0.2, 0.1, 0.1), p_v=(0.1, 0.3, 0.35, 0.25)),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def scaled(w: Workload, max_tensor_elems: int, max_tensors: int) -> Workload:
    """A reduced copy for CPU-sized tests: same recipe, fewer and smaller tensors (ragged sizes kept ragged)."""
    ts = []
    for name, n in w.tensors[:max_tensors]:
        if n > max_tensor_elems:
            n = max_tensor_elems + (n % 977)  # keep an irregular tail
        ts.append((name, n))
    return Workload(w.cfg, w.name + "-scaled", ts, w.K, w.grad_dtype, w.steps, w.grad_kind, w.bits_m, w.bits_v,
                    w.p_m, w.p_v, w.transitions, dict(w.hparams))
