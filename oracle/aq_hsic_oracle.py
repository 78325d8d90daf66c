"""CPU oracle for the HSIC-based tensor sensitivity (TEST INFRASTRUCTURE, not product code; parity pinned by
tests/test_hsic_oracle_pins.py).

What it follows:
  - empirical HSIC (Section 3, "Hilbert-Schmidt Independence Criterion", Eq. 2):
        HSIC(A, B) = (K - 1)^-2 tr(K_A C K_B C),   [K_A]_ij = k_A(a_i, a_j),   C = I - (1/K) 1 1^T
    over K paired samples a_k (row k of A) and b_k (row k of B), with the RBF kernel "throughout";
  - sensitivity of a weight matrix (Section 4.1, Eq. 5):
        S = -alpha HSIC(X, Z) + beta HSIC(Z, Y)
    X = input hidden states of the backbone, Z = output hidden states of the matrix, Y = action labels.
Readings (the paper does not give them): the RBF kernel is k(a, a') = exp(-gamma ||a - a'||^2) and gamma is an
input (one per variable; a caller without a better idea passes 1 / median squared distance, `median_gamma`).

Plain numpy in float64, the definition written out: pairwise differences, the centering matrix as a matrix, two
matrix products and a trace.  Meant for K up to a few thousand.
"""
from __future__ import annotations

import numpy as np


def rbf_gram(A: np.ndarray, gamma: float) -> np.ndarray:
    """[K_A]_ij = exp(-gamma ||a_i - a_j||^2), float64 [K, K]."""
    A = np.asarray(A, dtype=np.float64)
    K = A.shape[0]
    G = np.empty((K, K), dtype=np.float64)
    for i in range(K):
        diff = A - A[i]
        G[i] = np.exp(-gamma * np.sum(diff * diff, axis=1))
    return G


def median_gamma(A: np.ndarray) -> float:
    """1 / median of the squared distances between distinct samples."""
    A = np.asarray(A, dtype=np.float64)
    K = A.shape[0]
    d2 = []
    for i in range(K):
        diff = A[i + 1:] - A[i]
        d2.append(np.sum(diff * diff, axis=1))
    return 1.0 / float(np.median(np.concatenate(d2)))


def hsic(A: np.ndarray, gamma_a: float, B: np.ndarray, gamma_b: float) -> float:
    K = A.shape[0]
    assert B.shape[0] == K and K >= 2
    KA, KB = rbf_gram(A, gamma_a), rbf_gram(B, gamma_b)
    C = np.eye(K) - np.ones((K, K)) / K
    return float(np.trace(KA @ C @ KB @ C)) / (K - 1) ** 2


def sensitivity(X, gamma_x, Z, gamma_z, Y, gamma_y, alpha: float, beta: float) -> float:
    return -alpha * hsic(X, gamma_x, Z, gamma_z) + beta * hsic(Z, gamma_z, Y, gamma_y)
