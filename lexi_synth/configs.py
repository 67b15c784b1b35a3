"""The synthetic MoE-stack workloads and their scaled-down test shapes.

Shapes follow the paper's Table 1 (layers, experts, baseline top-k, FFN dim)
for OLMoE-1B-7B, Qwen1.5-MoE-A2.7B, Mixtral-8x7B and DeepSeek-V2-Lite; hidden
sizes, SwiGLU and shared experts come from the public model cards of those
models.  Weights and activations are synthetic (see ``generator``).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np

from . import generator as g

SHARED_NONE = 0
SHARED_UNGATED = 1
SHARED_SIGMOID = 2


@dataclass(frozen=True)
class MoEConfig:
    name: str
    number: int                 # seed offset: seed = BASE_SEED + number
    L: int
    d: int
    E: int
    F: int
    dtype: str                  # 'f32' or 'bf16' (x, expert weights, SwiGLU intermediate)
    k_base: int
    k_min: int
    k_max: int
    budget: int                 # sum of the LExI-style k vector
    T_regimes: Tuple[int, ...]
    F_shared: int = 0
    shared_kind: int = SHARED_NONE
    zipf_s: float = 0.0         # > 0: per-expert router bias -s*ln(rank)
    fixed_kvec: Optional[Tuple[int, ...]] = None
    sigma_w: float = 0.02
    sigma_x: float = 1.0

    @property
    def seed(self) -> int:
        return g.BASE_SEED + self.number

    def k_uniform(self) -> np.ndarray:
        return np.full(self.L, self.k_base, dtype=np.int32)

    def k_lexi(self) -> np.ndarray:
        """Static per-layer allocation k* = (k_1..k_L) with sum == budget."""
        if self.fixed_kvec is not None:
            return np.asarray(self.fixed_kvec, dtype=np.int32)
        return g.k_vector(self.seed, self.L, self.budget, self.k_min, self.k_max)

    def weight_bytes(self) -> int:
        es = 4 if self.dtype == "f32" else 2
        per_layer = 3 * self.E * self.d * self.F * es + 3 * self.d * self.F_shared * es + self.d * self.E * 4
        return self.L * per_layer


C1 = MoEConfig("c1_plumbing", 1, L=1, d=128, E=8, F=256, dtype="f32", k_base=2, k_min=2, k_max=2,
               budget=2, T_regimes=(64,))
C2 = MoEConfig("c2_olmoe", 2, L=16, d=2048, E=64, F=1024, dtype="bf16", k_base=8, k_min=2, k_max=8,
               budget=96, T_regimes=(4096,))
C3 = MoEConfig("c3_qwen15", 3, L=24, d=2048, E=60, F=1408, dtype="bf16", k_base=4, k_min=1, k_max=4,
               budget=72, T_regimes=(8192, 64), F_shared=5632, shared_kind=SHARED_SIGMOID)
# Mixtral-shaped: the paper's sensitivity figure finds the early layers the
# robust ones, so the k=1 half is the first half.
C4 = MoEConfig("c4_mixtral", 4, L=32, d=4096, E=8, F=14336, dtype="bf16", k_base=2, k_min=1, k_max=2,
               budget=48, T_regimes=(4096, 32), fixed_kvec=tuple([1] * 16 + [2] * 16))
C5 = MoEConfig("c5_dsv2lite", 5, L=26, d=2048, E=64, F=1408, dtype="bf16", k_base=6, k_min=2, k_max=6,
               budget=104, T_regimes=(1, 16, 64, 256), F_shared=2816, shared_kind=SHARED_UNGATED, zipf_s=1.1)

# The two remaining rows of the paper's Table 1, as shape variants for the throughput sweeps (hidden sizes and the
# shared experts of the DeepSeek-VL2 language model from the public model cards; 11 of its 12 layers are MoE layers,
# which is what the budgets 44 and 55 of the paper's figures are multiples of).
C6 = MoEConfig("c6_minicpm", 6, L=40, d=2304, E=8, F=5760, dtype="bf16", k_base=2, k_min=1, k_max=2,
               budget=60, T_regimes=(4096,))
C7 = MoEConfig("c7_vl2tiny", 7, L=11, d=1280, E=64, F=896, dtype="bf16", k_base=6, k_min=2, k_max=6,
               budget=44, T_regimes=(4096,), F_shared=1792, shared_kind=SHARED_UNGATED)

CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5, C6, C7)}


def mini(cfg: MoEConfig, L: int = 2, d: int = 256, F: int = 384, F_shared: Optional[int] = None) -> MoEConfig:
    """Same routing structure (E, k range, shared kind, bias) at a size the CPU oracle finishes in seconds."""
    fs = (F_shared if F_shared is not None else (2 * F if cfg.F_shared else 0))
    budget = max(L * cfg.k_min, min(L * cfg.k_max, round(cfg.budget * L / cfg.L)))
    fixed = None
    if cfg.fixed_kvec is not None:
        fixed = tuple([cfg.k_min] * (L // 2) + [cfg.k_max] * (L - L // 2))
        budget = sum(fixed)
    return replace(cfg, name=cfg.name + "_mini", L=L, d=d, F=F, F_shared=fs, budget=budget, fixed_kvec=fixed)


def pruned(cfg: MoEConfig, inter: float = 0.0, intra: float = 0.0) -> MoEConfig:
    """The SHAPE of an expert-pruned model (the paper's comparison methods, Sec. 3 "Inter and Intra Expert Pruning"):
    inter-pruning removes a fraction of the experts (and their router columns) and keeps k; intra-pruning shrinks
    every expert's FFN width.  Which experts or channels go is decided from calibration data in those methods and
    is not modelled: the weights stay synthetic, only the shapes change.  E' = floor(E (1 - inter));
    F' = F (1 - intra) rounded down to a multiple of 64 (the kernels' granularity)."""
    E = max(1, int(cfg.E * (1.0 - inter)))
    F = max(64, int(cfg.F * (1.0 - intra)) // 64 * 64)
    k_base = min(cfg.k_base, E)
    tag = (f"_inter{int(round(inter * 1000))}" if inter else "") + (f"_intra{int(round(intra * 1000))}" if intra else "")
    return replace(cfg, name=cfg.name + tag, E=E, F=F, k_base=k_base, k_max=min(cfg.k_max, E), k_min=min(cfg.k_min, E),
                   budget=min(cfg.budget, cfg.L * min(cfg.k_max, E)))
