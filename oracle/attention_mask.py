"""Unfactorized strided sparse self-attention pattern (Sec. 3.3) and its FLOP ratio
Q_atten (App. "FLOP Calculation", table of attention patterns).

TEST INFRASTRUCTURE ONLY (see the package docstring).

Reading: the set S_i is printed as the intersection of the window of the previous l
positions with the positions a multiple of l back, which would leave position i alone;
the text (previous l locations as well as every l-th location) and the figure describe
the union, and only the union reproduces the printed ratios (12.07 % for l = 128,
22.03 % for l = 256 at L = 1024, counted against all L * L pairs).

    S_i = { max(i - l + 1, 0), ..., i }  union  { j <= i : (i - j) mod l = 0 }
"""
from __future__ import annotations

import numpy as np


def strided_mask(L: int, l: int) -> np.ndarray:
    """[L x L] uint8, entry (i, j) = 1 iff output i attends to position j."""
    if L < 1 or l < 1:
        raise ValueError("L and l must be positive")
    m = np.zeros((L, L), dtype=np.uint8)
    for i in range(L):
        for j in range(max(i - l + 1, 0), i + 1):
            m[i, j] = 1
        for j in range(i + 1):
            if (i - j) % l == 0:
                m[i, j] = 1
    return m


def q_atten(L: int, l: int) -> float:
    """Share of the L * L query-key pairs the pattern keeps."""
    return float(strided_mask(L, l).sum(dtype=np.int64)) / float(L * L)
