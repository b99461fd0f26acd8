"""Sparsity Variation and update-fraction schedules (Sec. 3.1, Sec. 3.2).

Readings taken where the printed equations cannot be used literally:
  * The two cubic formulas of Sec. 3.1 put the floor around t / (N * Delta), which is
    zero throughout the phase; the text speaks of N stages, one every Delta steps, so the
    stage index is k = min(N, floor(t_phase / Delta)) and the cubic acts on k / N.
  * Evaluated as printed the warm-up would start at 100 % *sparsity*, while the text
    says a dense model becomes sparse.  The formulas are therefore read in density
    d = 1 - S:  warm-up      d = d_min + (1 - d_min) (1 - k/N)^3
                restoration  d = 1 + (d_min - 1) (1 - k/N)^3
  * Between the phases d = d_min; after restoration d = 1.
  * Stage k = 0 lasts for the first Delta steps of its phase (first change at Delta).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List


@dataclass
class ScheduleCfg:
    """Hyper-parameters of Table "Private hyperparameters of MST" (defaults are the paper's)."""
    S_M: float = 0.96          # maximum sparsity
    N: int = 5                 # number of sparsity stages
    Delta_W: int = 2000        # pruning frequency (warm-up)
    T_U: int = 100000          # ultra-sparsification duration
    Delta_R: int = 2000        # growing frequency (restoration)
    zeta: List[float] = field(default_factory=lambda: [0.3] * 6)  # zeta_1 .. zeta_{N+1}

    @property
    def T_W(self) -> int:
        return self.N * self.Delta_W

    @property
    def T_R(self) -> int:
        return self.N * self.Delta_R


def density(cfg: ScheduleCfg, t: int) -> float:
    """Target density 1 - S_t at training step t (Sec. 3.1, both display equations)."""
    d_min = 1.0 - cfg.S_M
    if t < 0:
        raise ValueError("step must be >= 0")
    if t < cfg.T_W:
        k = min(cfg.N, t // cfg.Delta_W)
        return d_min + (1.0 - d_min) * (1.0 - k / cfg.N) ** 3
    if t < cfg.T_W + cfg.T_U:
        return d_min
    if t < cfg.T_W + cfg.T_U + cfg.T_R:
        k = min(cfg.N, (t - cfg.T_W - cfg.T_U) // cfg.Delta_R)
        return 1.0 + (d_min - 1.0) * (1.0 - k / cfg.N) ** 3
    return 1.0


def zeta_boundaries(cfg: ScheduleCfg) -> List[int]:
    """T_0 .. T_{N+1} of the piecewise cosine (Sec. 3.2, text below the zeta equation)."""
    b = [0, cfg.T_W + cfg.T_U]
    for j in range(1, cfg.N + 1):
        b.append(cfg.T_W + cfg.T_U + j * cfg.Delta_R)
    return b


def zeta(cfg: ScheduleCfg, t: int) -> float:
    """Topology update fraction zeta_t (Sec. 3.2, piecewise decaying cosine annealing).

    Period i covers [T_{i-1}, T_i) with magnitude zeta_i; after the last period the
    layer is dense and nothing is updated (0).
    """
    if t < 0:
        raise ValueError("step must be >= 0")
    b = zeta_boundaries(cfg)
    if len(cfg.zeta) != cfg.N + 1:
        raise ValueError("need N + 1 zeta magnitudes")
    for i in range(1, len(b)):
        if b[i - 1] <= t < b[i]:
            return 0.5 * cfg.zeta[i - 1] * (1.0 + math.cos(math.pi * (t - b[i - 1]) / (b[i] - b[i - 1])))
    return 0.0
