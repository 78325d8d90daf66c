"""Pins of the HSIC oracle (oracle/aq_hsic_oracle.py) against things other than itself: hand-worked values, the
population form of the appendix evaluated on the samples (another formula for the same number), scipy's pairwise
distances, and the properties a dependence measure has.  No GPU."""
import math
import os

import numpy as np
from scipy.spatial.distance import cdist

import aq_workloads as wl
from oracle import aq_hsic_oracle as ho

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hsic_example.txt")


def golden():
    return {l.split()[0]: float(l.split()[1]) for l in open(GOLDEN) if l.strip() and not l.startswith("#")}


def test_hand_worked_values():
    g = golden()
    ln2 = math.log(2.0)
    A = np.array([[0.0], [1.0]]); B = np.array([[0.0], [2.0]])
    assert abs(ho.hsic(A, ln2, B, ln2) - g["hsic_two_samples"]) < 1e-15
    A3 = np.array([[0.0], [1.0], [2.0]])
    assert abs(ho.hsic(A3, ln2, A3, ln2) - g["hsic_three_samples"]) < 1e-15


def test_gram_matrix_against_scipy():
    X, Z, _ = wl.draw_hsic_inputs(40, 24, 16, 3, 81)
    for A, gamma in ((X, 0.02), (Z, 0.05)):
        want = np.exp(-gamma * cdist(A.astype(np.float64), A.astype(np.float64), "sqeuclidean"))
        assert np.allclose(ho.rbf_gram(A, gamma), want, rtol=1e-12, atol=0)
    # 1 / median squared distance
    d2 = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")[np.triu_indices(40, 1)]
    assert abs(ho.median_gamma(X) * np.median(d2) - 1.0) < 1e-12


def test_equals_the_population_form_evaluated_on_the_samples():
    """Appendix "HSIC": E[k_A k_B] + E[k_A] E[k_B] - 2 E[E'[k_A] E'[k_B]] with sample means in place of the
    expectations is K^-2 tr(K_A C K_B C): the estimator times ((K-1)/K)^2."""
    X, Z, Y = wl.draw_hsic_inputs(64, 20, 12, 4, 82)
    K = 64
    for (A, ga, B, gb) in ((X, 0.03, Z, 0.06), (Z, 0.06, Y, 0.4)):
        KA, KB = ho.rbf_gram(A, ga), ho.rbf_gram(B, gb)
        v = (KA * KB).mean() + KA.mean() * KB.mean() - 2.0 * (KA.mean(axis=1) * KB.mean(axis=1)).mean()
        assert abs(ho.hsic(A, ga, B, gb) - v * K * K / (K - 1) ** 2) < 1e-14


def test_properties():
    X, Z, Y = (a.astype(np.float64) for a in wl.draw_hsic_inputs(96, 16, 16, 4, 83))
    gx, gz = ho.median_gamma(X), ho.median_gamma(Z)
    h = ho.hsic(X, gx, Z, gz)
    assert abs(h - ho.hsic(Z, gz, X, gx)) < 1e-15                       # symmetric in its two arguments
    assert abs(h - ho.hsic(X + 3.0, gx, Z - 1.0, gz)) < 1e-12           # the RBF kernel sees differences only
    perm = np.random.default_rng(0).permutation(96)
    assert abs(h - ho.hsic(X[perm], gx, Z[perm], gz)) < 1e-14           # the order of the paired samples is free
    # dependence, by the permutation test built on this statistic (re-pairing the samples at random draws from the
    # null distribution of independence; the empirical estimator is what Section 3, "HSIC", defines): Z is a noisy
    # linear map of X, so the statistic of the true pairing lies above that of every one of 50 random re-pairings
    # (level 1/51); for an independent redraw of Z the true pairing is exchangeable with the re-pairings and does not
    rng = np.random.default_rng(1)
    null = [ho.hsic(X, gx, Z[rng.permutation(96)], gz) for _ in range(50)]
    assert h > max(null)
    _, Z2, _ = wl.draw_hsic_inputs(96, 16, 16, 4, 84)
    Z2 = Z2.astype(np.float64)
    g2 = ho.median_gamma(Z2)
    h_ind = ho.hsic(X, gx, Z2, g2)
    null2 = [ho.hsic(X, gx, Z2[rng.permutation(96)], g2) for _ in range(50)]
    assert 0.0 < h_ind < max(null2)                                     # (the estimator has a bias of order 1/K)
    assert ho.hsic(X, gx, X, gx) > h
    # constant variable: its centred kernel matrix vanishes
    assert abs(ho.hsic(X, gx, np.ones((96, 2)), 1.0)) < 1e-15
    # Eq. 5
    gy = ho.median_gamma(Y)
    s = ho.sensitivity(X, gx, Z, gz, Y, gy, 0.25, 2.0)
    assert abs(s - (-0.25 * h + 2.0 * ho.hsic(Z, gz, Y, gy))) < 1e-15
