"""Gaussian-sketch rank-1 deflation (Section 3.1, "Plug-in", Eq. 13), written out in numpy fp64.

TEST INFRASTRUCTURE ONLY.  For each of r ranks, with the caller's sketch vector s:
    Q = (W W^T)^it W s,  U = Q / |Q|,  Sigma = |Q^T W| / |Q|,  V = Q^T W / |Q^T W|,  W <- W - U Sigma V.
The powers are taken literally (no renormalisation between iterations)."""
from __future__ import annotations

import numpy as np


def sketch_lowrank(W: np.ndarray, r: int, it: int, sketch: np.ndarray):
    """W [rows, cols], sketch [r, cols].  Returns (U [r, rows], sigma [r], V [r, cols], residual [rows, cols]) in float64."""
    W = np.array(W, dtype=np.float64)
    S = np.asarray(sketch, dtype=np.float64)
    rows, cols = W.shape
    assert S.shape == (r, cols)
    U = np.zeros((r, rows))
    V = np.zeros((r, cols))
    sigma = np.zeros(r)
    for rho in range(r):
        Q = W @ S[rho]
        for _ in range(it):
            Q = W @ (W.T @ Q)
        nq = np.linalg.norm(Q)
        if nq == 0.0:
            continue                      # the matrix has run out of rank: zero vectors, Sigma = 0
        P = Q @ W                         # Q^T W
        npn = np.linalg.norm(P)
        U[rho] = Q / nq
        sigma[rho] = npn / nq
        if npn > 0.0:
            V[rho] = P / npn
        W = W - sigma[rho] * np.outer(U[rho], V[rho])
    return U, sigma, V, W
