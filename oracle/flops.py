"""Theoretical FLOP counts (App. "FLOP Calculation").

TEST INFRASTRUCTURE ONLY (see the package docstring).

Readings:
  * The "reduce" term is printed with the embedding size times L * L * D_head, which
    would be the head count times too large (103 GFLOP per block for GPT-2 small); it is
    read as (number of heads) * L * L * D_head = L * L * N_embd, the cost of applying the
    attention weights to the values.  With it, and the vocabulary padded to 50304 as in
    the code base the public hyper-parameters come from, the counts reproduce the FLOPs
    column of the main results table for the static-sparse 80 % row (267.7 G) and the
    Tiny row (212.7 G); the dense row comes out as 874.8 G where the table prints 847.8 G
    (two digits exchanged).
  * Every fully-connected term carries (1 - S), the output layer included, as printed.
  * Backward = 2 x forward, training = forward + backward.
"""
from __future__ import annotations

from typing import Dict, Sequence, Tuple


def fc_forward(shapes: Sequence[Tuple[int, int]], sparsity: Sequence[float]) -> float:
    """Eq. (1): sum_l (1 - S_l)(2 I_l - 1) O_l, per token.  shapes = [(O_l, I_l)]."""
    if len(shapes) != len(sparsity):
        raise ValueError("one sparsity per layer")
    return sum((1.0 - s) * (2 * I - 1) * O for (O, I), s in zip(shapes, sparsity))


def transformer(L: int, n_embd: int, d_ffw: int, d_vocab: int, n_layers: int,
                S: float, q_atten: float) -> Dict[str, float]:
    """The seven terms of the appendix for one sequence of L tokens, and their totals."""
    kqv = (1.0 - S) * L * ((2 * n_embd - 1) * 3 * n_embd)
    scores = q_atten * 2 * L * L * n_embd
    reduce_ = q_atten * 2 * L * L * n_embd
    proj = (1.0 - S) * L * ((2 * n_embd - 1) * n_embd)
    ffw1 = (1.0 - S) * L * ((2 * n_embd - 1) * d_ffw)
    ffw2 = (1.0 - S) * L * ((2 * d_ffw - 1) * n_embd)
    lm = (1.0 - S) * L * ((2 * n_embd - 1) * d_vocab)
    atten = kqv + scores + reduce_ + proj
    mlp = ffw1 + ffw2
    forward = n_layers * (atten + mlp) + lm
    return {"kqv": kqv, "scores": scores, "reduce": reduce_, "proj": proj, "ffw1": ffw1,
            "ffw2": ffw2, "lm": lm, "forward": forward, "backward": 2.0 * forward,
            "total": 3.0 * forward}
