"""The four matrix products of a masked fully-connected layer, as their definitions.

A layer holds W [O, I] and a binary mask M [O, I]; its effective weight is
W * M (Algorithm 1, last line).  With X [T, I] the layer input and dY [T, O] the
gradient arriving at its output (App. "FLOP Calculation": forward Eq. (1), backward
counted as twice the forward, i.e. one product for the input gradient and one for
the weight gradient):

    forward         Y  = X  (W*M)^T                      [T, O]
    input gradient  dX = dY (W*M)                        [T, I]
    weight gradient dW = (dY^T X) * M, listed for the active positions only,
                         in ascending flat index o*I + i [nnz]
    dense gradient  G  = dY^T X (all positions; the score of the gradient-based
                         growth in Algorithm 1)          [O, I]

Inputs are widened exactly to float64; every result is float64 and is rounded by the
caller if it wants fp32.  numpy's matmul is the only primitive.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def effective_weight(W, M) -> np.ndarray:
    return _f64(W) * (np.asarray(M) != 0)


def fc_fwd(X, W, M) -> np.ndarray:
    return _f64(X) @ effective_weight(W, M).T


def fc_bwd_input(dY, W, M) -> np.ndarray:
    return _f64(dY) @ effective_weight(W, M)


def dense_grad(dY, X) -> np.ndarray:
    return _f64(dY).T @ _f64(X)


def fc_bwd_weight(dY, X, M) -> np.ndarray:
    G = dense_grad(dY, X)
    return G[np.asarray(M) != 0]          # boolean indexing walks row-major = ascending flat index


# --- one output element at a time, for spot checks at sizes where the full
# --- product is too slow -----------------------------------------------------

def fc_fwd_at(X, W, M, t: int, o: int) -> float:
    return float(np.dot(_f64(X[t]), effective_weight(W[o], M[o])))


def fc_bwd_input_at(dY, W, M, t: int, i: int) -> float:
    return float(np.dot(_f64(dY[t]), effective_weight(W[:, i], M[:, i])))


def dense_grad_at(dY, X, o: int, i: int) -> float:
    return float(np.dot(_f64(dY[:, o]), _f64(X[:, i])))
