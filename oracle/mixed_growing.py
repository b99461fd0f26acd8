"""Mixed-Growing topology update for one layer (Sec. 3.2, Algorithm 1), step by step.

Readings taken where Algorithm 1 is silent or cannot be used as printed:
  counts   * the target active count is the nearest integer to d' * N (halves up);
           * N_prune = floor(zeta * nnz) with nnz the layer's actual active count;
           * N_grow = N_prune + (nnz' - nnz): the printed "+ (s' - s) N" has the right
             sign only when s is read as density (same slip as in Sec. 3.1); this is the
             only choice for which the layer lands on its target;
           * if that N_grow is negative nothing grows and exactly nnz - nnz' are pruned;
             if it exceeds the inactive positions, all of them grow and the prune count
             is reduced to keep the target;
           * N_rand = floor(N_grow * R), N_grad = N_grow - N_rand as printed.
  prune    ArgTopK(-|theta * M|) is taken over ACTIVE positions only (an inactive
           position has |theta * M| = 0 and would otherwise always win).
  grow     candidates are the positions inactive before this update; the positions
           just pruned are active before the update and so cannot regrow in the same
           update.  Random growth draws from the candidates not chosen by gradient.
  ties     every selection is a total order: (score, flat index) with the lower flat
           index first.  |.| is compared on fp32 values (bit pattern with the sign bit
           cleared, which orders finite non-negative floats).  Inputs must be finite.
  RandK    "uniformly at random without replacement" is realised by giving flat index f
           the key SplitMix64(seed)[f] -- the (f+1)-th output of the SplitMix64
           generator started at state `seed` (Steele, Lea, Flood 2014) -- and taking
           the N_rand candidates with the smallest (key, f).
  values   theta <- theta * M: pruned weights become 0; grown weights start at 0.
  variant  the table of topology evolution schemes lists one other prune criterion,
           min(|theta| + lambda |grad|); `prune_lambda` > 0 selects it (the gradient is the
           same dense gradient that scores growth; lambda is the caller's, the paper gives
           no value).  The score is formed in fp32: the product is rounded, then the sum.
           lambda = 0 is the paper's own criterion.
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np

_U64 = np.uint64


def target_count(n_total: int, d_target: float) -> int:
    return int(math.floor(float(d_target) * n_total + 0.5))


def counts(n_total: int, nnz: int, d_target: float, zeta: float, R: float) -> Dict[str, int]:
    """Algorithm 1, the four count lines, with the clamp rules listed in the header."""
    nnz_t = target_count(n_total, d_target)
    n_prune = int(math.floor(float(zeta) * nnz))
    n_grow = n_prune + (nnz_t - nnz)
    if n_grow < 0:
        n_prune, n_grow = nnz - nnz_t, 0
    if n_grow > n_total - nnz:
        n_grow = n_total - nnz
        n_prune = n_grow - (nnz_t - nnz)
    n_rand = int(math.floor(n_grow * float(R)))
    n_grad = n_grow - n_rand
    return dict(nnz_target=nnz_t, n_prune=n_prune, n_grow=n_grow, n_rand=n_rand, n_grad=n_grad)


def abs_bits(a) -> np.ndarray:
    """fp32 magnitude as an integer that orders like |a| for finite a (+0 == -0)."""
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def randk_key(seed: int, f) -> np.ndarray:
    """SplitMix64(seed)[f] for an array of flat indices f (uint64 arithmetic mod 2^64)."""
    f = np.asarray(f, dtype=_U64)
    with np.errstate(over="ignore"):
        z = _U64(seed & 0xFFFFFFFFFFFFFFFF) + (f + _U64(1)) * _U64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        z = z ^ (z >> _U64(31))
    return z


def prune_score_bits(w, g, prune_lambda: float) -> np.ndarray:
    """Integer that orders like the prune score |w| + lambda |g| (fp32, two roundings)."""
    if prune_lambda == 0.0:
        return abs_bits(w)
    a = np.abs(np.ascontiguousarray(w, dtype=np.float32))
    b = np.float32(prune_lambda) * np.abs(np.ascontiguousarray(g, dtype=np.float32))
    with np.errstate(over="ignore"):
        return (a + b.astype(np.float32)).astype(np.float32).view(np.uint32)


def update(W, M, G, d_target: float, zeta: float, R: float, seed: int,
           prune_lambda: float = 0.0) -> Dict[str, object]:
    """One Mixed-Growing update of a layer.

    W [O, I] fp32 weights (zero at inactive positions), M [O, I] 0/1 mask, G [O, I]
    fp32 dense weight gradient (the score buffer).  Returns the new mask and weights
    and the three index sets (sorted flat indices).
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    G = np.ascontiguousarray(G, dtype=np.float32)
    Mb = np.asarray(M).reshape(-1) != 0
    n_total = Mb.size
    active = np.flatnonzero(Mb)
    inactive = np.flatnonzero(~Mb)
    c = counts(n_total, active.size, d_target, zeta, R)

    # prune: the n_prune active weights with the smallest (score, f), score = |w| (+ lambda |g|)
    wkey = prune_score_bits(W.reshape(-1)[active], G.reshape(-1)[active], prune_lambda)
    order = np.lexsort((active, wkey))
    i_prune = np.sort(active[order[: c["n_prune"]]])

    # gradient growth: the n_grad candidates with the largest |g|, lowest f on ties
    gkey = abs_bits(G.reshape(-1)[inactive]).astype(np.int64)
    order = np.lexsort((inactive, -gkey))
    i_grad = np.sort(inactive[order[: c["n_grad"]]])

    # random growth among the remaining candidates: smallest (SplitMix64 key, f)
    rest = np.setdiff1d(inactive, i_grad, assume_unique=True)
    rkey = randk_key(seed, rest)
    order = np.lexsort((rest, rkey))
    i_rand = np.sort(rest[order[: c["n_rand"]]])

    M_new = Mb.copy()
    M_new[i_prune] = False
    M_new[i_grad] = True
    M_new[i_rand] = True
    W_new = (W.reshape(-1) * Mb * M_new).astype(np.float32)   # pruned -> 0, grown start at 0
    W_new[~M_new] = 0.0                                        # also clears -0.0 and stale values
    W_new[i_grad] = 0.0
    W_new[i_rand] = 0.0
    return dict(
        M=M_new.astype(np.uint8).reshape(np.asarray(M).shape),
        W=W_new.reshape(W.shape),
        prune=i_prune, grad=i_grad, rand=i_rand, counts=c,
    )
