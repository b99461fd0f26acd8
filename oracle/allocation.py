"""Per-layer density allocation by the Erdos-Renyi strategy (Sec. 3.2, the sentence that
derives each layer's sparsity from the network's; the strategy is the one of the sparse
evolutionary training paper it cites).

TEST INFRASTRUCTURE ONLY (see the package docstring).

A layer with I inputs and O outputs gets density

    d_l = min(1, eps * (I_l + O_l) / (I_l * O_l))

and eps is the number for which the layers together hold the network's budget,

    sum_l d_l * N_l = d * sum_l N_l,      N_l = I_l * O_l.

Readings (the paper gives one sentence and a citation):
  * which layers take part is the caller's list;
  * a layer whose share would exceed 1 is dense and the rest is solved again, until no
    further layer saturates (the usual treatment of this rule);
  * the result is a real-valued density per layer; turning it into a count is the count
    rule of Algorithm 1's first lines (mixed_growing.counts).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def erdos_renyi_density(shapes: Sequence[Tuple[int, int]], d: float) -> List[float]:
    """shapes = [(O_l, I_l)], d = network density in [0, 1]  ->  [d_l]."""
    if not shapes:
        raise ValueError("need at least one layer")
    if not (0.0 <= d <= 1.0):
        raise ValueError("density must be in [0, 1]")
    for O, I in shapes:
        if O < 1 or I < 1:
            raise ValueError("layer dimensions must be positive")
    n = [float(O) * float(I) for O, I in shapes]
    budget = d * sum(n)
    dense = [False] * len(shapes)
    while True:
        free = [l for l in range(len(shapes)) if not dense[l]]
        if not free:
            return [1.0] * len(shapes)
        # eps * (I + O) / (I * O) * N_l = eps * (I + O)
        eps = (budget - sum(n[l] for l in range(len(shapes)) if dense[l])) / sum(
            float(shapes[l][0] + shapes[l][1]) for l in free)
        over = [l for l in free if eps * (shapes[l][0] + shapes[l][1]) / n[l] > 1.0]
        if not over:
            return [1.0 if dense[l] else eps * (shapes[l][0] + shapes[l][1]) / n[l]
                    for l in range(len(shapes))]
        for l in over:
            dense[l] = True
