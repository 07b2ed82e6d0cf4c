"""fp64 oracle of the channel-mixing linear between the pooling and the contraction.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Section 4.1 (the paragraph before Algorithm 2): after the messages are summed over the
neighbours, the channels k belonging to one order l are mixed linearly once more before the
symmetric contraction.  For every atom i, output channel k', order l and m

    Y[i,k',(l,m)] = sum_k W[l,k,k'] * X[i,k,(l,m)]

i.e. one K_in x K_out matrix per order l, shared by the 2l+1 components m of that order (a
matrix that depended on m would break equivariance).  Component index l*l + l + m as
everywhere else.  Readings: no bias (a bias is only equivariant for l = 0 and the paper
mentions none), no normalisation factor inside the operation (a caller folds 1/sqrt(K_in)
into W if wanted), K_in and K_out may differ.
The backward functions are the analytic derivatives.
"""
from __future__ import annotations

import numpy as np


def order_of_component(l_max: int) -> np.ndarray:
    return np.concatenate([np.full(2 * l + 1, l) for l in range(l_max + 1)])


def forward(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """X: (N, K_in, (l_max+1)^2), W: (l_max+1, K_in, K_out) -> Y: (N, K_out, (l_max+1)^2)."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    l_of = order_of_component(W.shape[0] - 1)
    assert X.shape[2] == l_of.size and X.shape[1] == W.shape[1]
    Y = np.zeros((X.shape[0], W.shape[2], X.shape[2]))
    for c, l in enumerate(l_of):
        Y[:, :, c] = X[:, :, c] @ W[l]
    return Y


def backward(X: np.ndarray, W: np.ndarray, dY: np.ndarray):
    """Gradients of sum(dY * Y) with respect to X and W."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    l_of = order_of_component(W.shape[0] - 1)
    dX = np.zeros_like(X)
    dW = np.zeros_like(W)
    for c, l in enumerate(l_of):
        dX[:, :, c] = dY[:, :, c] @ W[l].T
        dW[l] += X[:, :, c].T @ dY[:, :, c]
    return dX, dW
