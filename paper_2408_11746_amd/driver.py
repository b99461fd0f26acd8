"""Topology schedule over a set of layers: which step updates, with which targets.

Orchestration only: every decision (is this an update step, the density and update fraction,
the layers' shares, the per-layer seed, the counts) is a host call of the library, every device
step runs in the library; this file holds no arithmetic of the method.

At a step t that is a positive multiple of the update interval Delta_t (Table "Private
hyperparameters of MST": 100) the network density d_t and update fraction zeta_t of
Sec. 3.1 / 3.2 are evaluated, d_t is spread over the layers by the Erdos-Renyi strategy
(Sec. 3.2) and every layer takes one Mixed-Growing update (Algorithm 1) towards its share.
Once the schedule is dense and zeta_t is 0 nothing is left to do and the step is skipped.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from . import binding as B


class TopologyDriver:
    def __init__(self, layers: Sequence[B.Layer], cfg: B.ScheduleCfg, delta_t: int = 100,
                 rand_ratio: float = 0.25, seed: int = 0, allocation: str = "erdos_renyi"):
        if delta_t < 1:
            raise ValueError("delta_t must be positive")
        B.mst_update_due(0, delta_t)                    # the library's own argument check
        if allocation not in ("erdos_renyi", "uniform"):
            raise ValueError("allocation is 'erdos_renyi' or 'uniform'")
        self.layers = list(layers)
        self.cfg, self.delta_t, self.rand_ratio, self.seed = cfg, int(delta_t), float(rand_ratio), int(seed)
        self.allocation = allocation
        self.shapes = [(l.O, l.I) for l in self.layers]

    def is_update_step(self, step: int) -> bool:
        return B.mst_update_due(step, self.delta_t)

    def targets(self, step: int):
        """(d_t, zeta_t, [d_l]) at a step."""
        d, z = B.mst_schedule_density(self.cfg, step)
        if self.allocation == "uniform":
            return d, z, [d] * len(self.layers)
        return d, z, B.mst_erdos_renyi_density(self.shapes, d)

    def layer_seed(self, step: int, index: int) -> int:
        """Seed of the random growth of layer `index` at `step`: distinct per (step, layer)."""
        return B.mst_update_seed(self.seed, step, len(self.layers), index)

    def _idle(self, d_layers, z) -> bool:
        if z != 0.0:
            return False
        return all(B.mst_update_counts(O * I, l.nnz, dl, 0.0, 0.0)["nnz_after"] == l.nnz
                   for l, (O, I), dl in zip(self.layers, self.shapes, d_layers))

    def update_from_scores(self, step: int, scores: Sequence, ws, stream=None) -> Optional[List[dict]]:
        """One update of every layer from given score buffers; None when the step has none."""
        if not self.is_update_step(step):
            return None
        _, z, d_layers = self.targets(step)
        if self._idle(d_layers, z):
            return None
        return [B.mst_mask_update_from_scores(l, G, dl, z, self.rand_ratio, self.layer_seed(step, k), ws, stream)
                for k, (l, G, dl) in enumerate(zip(self.layers, scores, d_layers))]

    def update(self, step: int, dYs: Sequence, Xs: Sequence, T: int, ws, act: int = B.MST_F32,
               stream=None) -> Optional[List[dict]]:
        """The same with the scores computed from each layer's dY and X."""
        if not self.is_update_step(step):
            return None
        _, z, d_layers = self.targets(step)
        if self._idle(d_layers, z):
            return None
        return [B.mst_mask_update(l, dY, X, T, dl, z, self.rand_ratio, self.layer_seed(step, k), ws, act, stream)
                for k, (l, dY, X, dl) in enumerate(zip(self.layers, dYs, Xs, d_layers))]

    def update_with_weight_gradient(self, step: int, dYs: Sequence, Xs: Sequence, dWs: Sequence, T: int, ws,
                                    act: int = B.MST_F32, stream=None) -> Optional[List[dict]]:
        """On an update step: every layer's weight gradient (into dWs, at the positions active
        before the update) and its update from one dense gradient per layer.  None when the
        step has no update; the caller then runs the ordinary weight gradient."""
        if not self.is_update_step(step):
            return None
        _, z, d_layers = self.targets(step)
        if self._idle(d_layers, z):
            return None
        return [B.mst_sparse_fc_bwd_weight_update(l, dY, X, dW, T, dl, z, self.rand_ratio, self.layer_seed(step, k), ws,
                                                  act, stream)
                for k, (l, dY, X, dW, dl) in enumerate(zip(self.layers, dYs, Xs, dWs, d_layers))]
