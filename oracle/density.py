"""Spectral density and moment estimates from stochastic Lanczos quadrature.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Each probe's Lanczos run
yields nodes theta_i (Ritz values) and weights w_i (squared first eigenvector
components, Table 2 of the paper) of a discrete measure that matches the
moments of the spectral density seen from that probe.  The smoothed density the
paper plots is that measure broadened with a Gaussian and averaged over the
probes; with Rademacher probes the mean of q^T H^p q estimates tr(H^p)/n.
"""
from __future__ import annotations

import numpy as np


def smoothed_density(ritz, weights, m_eff, sigma, grid):
    """ritz, weights: [n_probes, m]; only the first m_eff[p] entries of row p
    are used.  Returns rho[len(grid)] = mean_p sum_i w_pi N(t; theta_pi, sigma^2)."""
    ritz, weights = np.atleast_2d(ritz), np.atleast_2d(weights)
    grid = np.asarray(grid, dtype=np.float64)
    rho = np.zeros_like(grid)
    for p in range(ritz.shape[0]):
        for i in range(int(m_eff[p])):
            z = (grid - ritz[p, i]) / sigma
            rho += weights[p, i] * np.exp(-0.5 * z * z) / (sigma * np.sqrt(2.0 * np.pi))
    return rho / ritz.shape[0]


def moments(ritz, weights, m_eff, n_moments):
    """mu_p = mean over probes of sum_i w_i theta_i^p, p = 0..n_moments-1:
    the quadrature estimate of tr(H^p)/n."""
    ritz, weights = np.atleast_2d(ritz), np.atleast_2d(weights)
    mu = np.zeros(n_moments)
    for p in range(ritz.shape[0]):
        k = int(m_eff[p])
        for q in range(n_moments):
            mu[q] += np.sum(weights[p, :k] * ritz[p, :k] ** q)
    return mu / ritz.shape[0]
