"""One-time host-side factorization of layer weights (eq. 1, 2 and 4 of the paper).

This is setup, not the hot path: it runs once per layer on the host with LAPACK (numpy) and
returns fp64 factor arrays in the orientation the library uses (see include/lrd.h):
``W[out,in] ~= U[out,r] @ V[r,in]`` and ``W[S,k,k,C] ~= P2 x G x P1``.
"""
from __future__ import annotations

import numpy as np


def svd_factors(W: np.ndarray, r: int):
    """Truncated SVD (eq. 2) with the singular values split evenly between the two factors:
    U = U_r sqrt(S_r), V = sqrt(S_r) V_r^T.  Returns (U [out,r], V [r,in], sigma)."""
    W = np.asarray(W, dtype=np.float64)
    u, s, vt = np.linalg.svd(W, full_matrices=False)
    if not 1 <= r <= s.shape[0]:
        raise ValueError("rank out of range")
    root = np.sqrt(s[:r])
    return u[:, :r] * root[None, :], root[:, None] * vt[:r], s


def tucker2_factors(W: np.ndarray, r1: int, r2: int):
    """Tucker-2 by truncated higher-order SVD on the two channel modes (eq. 4).
    W [S,k,k,C] -> P1 [r1,C], G [r2,k,k,r1], P2 [S,r2]."""
    W = np.asarray(W, dtype=np.float64)
    S, k, k2, C = W.shape
    if k != k2 or not (1 <= r1 <= C and 1 <= r2 <= S):
        raise ValueError("bad shape or rank")
    lead_c = np.linalg.svd(W.reshape(-1, C).T, full_matrices=False)[0][:, :r1]   # C x r1
    lead_s = np.linalg.svd(W.reshape(S, -1), full_matrices=False)[0][:, :r2]     # S x r2
    core = np.tensordot(np.tensordot(lead_s.T, W, axes=(1, 0)), lead_c, axes=(3, 0))  # r2,k,k,r1
    return lead_c.T.copy(), core, lead_s.copy()
