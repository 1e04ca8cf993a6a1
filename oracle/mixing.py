"""Dense mixing-matrix model of DS-Sync (Sec. IV-B2) -- TEST INFRASTRUCTURE ONLY.

A second, brute-force statement of the method used to pin ``ds_oracle.c``:
iteration k is ``X_{k+1} = W_k X_k`` where ``W_k`` is the N-by-N matrix whose
entry (i, j) is ``1/|group|`` when workers i and j share a group in iteration
k and 0 otherwise.  Everything is numpy fp64 and O(N^2 P); use it for tiny N.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np


def groups_of(perm, off):
    """List of member lists, group k = perm[off[k]:off[k+1]]."""
    perm = np.asarray(perm)
    return [perm[off[k]:off[k + 1]].tolist() for k in range(len(off) - 1)]


def mixing_matrix(perm, off) -> np.ndarray:
    """``W_k`` of Sec. IV-B2 for one division of the workers."""
    N = len(perm)
    Wk = np.zeros((N, N), dtype=np.float64)
    for members in groups_of(perm, off):
        for i in members:
            for j in members:
                Wk[i, j] = 1.0 / len(members)
    return Wk


def step_dense(X: np.ndarray, G: np.ndarray, perm, off, lr: float) -> np.ndarray:
    """``W_k (X - lr G)``: local update of every worker, then group average."""
    Y = X.astype(np.float64) - float(np.float32(lr)) * G.astype(np.float64)
    return mixing_matrix(perm, off) @ Y


def product(matrices: Sequence[np.ndarray]) -> np.ndarray:
    """``W_{K-1} ... W_1 W_0`` -- later iterations multiply on the left."""
    N = matrices[0].shape[0]
    acc = np.eye(N)
    for Wk in matrices:
        acc = Wk @ acc
    return acc


def closed_form(x0: np.ndarray, deltas: Sequence[np.ndarray], matrices: Sequence[np.ndarray]) -> np.ndarray:
    """Replica stack after T iterations by the closed form of Sec. III-A step 4.

    ``x0`` is the shared initial model (length P), ``deltas[t]`` the N-by-P
    stack of local update vectors of iteration t, ``matrices[t]`` its ``W_t``.
    Row i of the result is ``w_0 + sum_t ( (W_{T-1} ... W_t) deltas[t] )_i``:
    the update of iteration t is averaged by every division from t onwards.
    """
    T = len(matrices)
    N = matrices[0].shape[0]
    out = np.tile(np.asarray(x0, dtype=np.float64), (N, 1))
    for t in range(T):
        out = out + product(matrices[t:]) @ np.asarray(deltas[t], dtype=np.float64)
    return out


def second_eigenvalue(M: np.ndarray) -> float:
    """Second largest eigenvalue modulus of a doubly stochastic matrix.

    For the product of one period of divisions this is Lemma 1's rho.
    """
    ev = np.sort(np.abs(np.linalg.eigvals(M)))[::-1]
    return float(ev[1]) if len(ev) > 1 else 0.0


def contraction_norm(M: np.ndarray) -> float:
    """``|| M - 11^T/N ||_2``: how much one application of ``M`` shrinks the
    part of a stack orthogonal to consensus.  Equals ``second_eigenvalue`` for
    symmetric ``M``; for a product of divisions it is the rigorous factor in
    ``|| M^k X - mean ||_F <= sigma^k || X ||_F``.
    """
    N = M.shape[0]
    return float(np.linalg.norm(M - np.ones((N, N)) / N, 2))
