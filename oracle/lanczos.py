"""Float64 Lanczos iteration and stochastic-Lanczos-quadrature read-out.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

`lanczos` follows the paper's Algorithm 2 in its order and notation: normalise
q_0; for each k apply the operator, subtract beta_{k-1} q_{k-1}, take
alpha_k = <q_k, r>, subtract alpha_k q_k, take beta_k = ||r||, stop if
beta_k < eps, else q_{k+1} = r / beta_k.  The full-orthogonalisation variant
(Section "Memory Compute trade off": the baseline that stores Q) is only named
in the paper; the reading used here: after the two three-term subtractions,
classical Gram-Schmidt of r against every stored q_0..q_k (c = Q^T r,
r -= Q c), repeated once more when the pass shrank ||r|| below 1/sqrt(2) of its
value before the pass; alpha_k is not corrected.

`slq_readout` follows Section "A note on numerical precision for the weight
value" / Table 2: solve the k x k tridiagonal eigenproblem exactly; Ritz values
ascending; one weight per Ritz value, the squared first component of the unit
eigenvector of T (the Gauss-quadrature weight, which is what sums to one as the
table's weights do).
"""
from __future__ import annotations

import numpy as np


def lanczos(apply_H, q0, m, reorth="none", tol=0.0, return_basis=False):
    """Returns (alpha[m_eff], beta[m_eff], m_eff[, Q[m_eff(+1), n]]).

    beta[k] is the norm computed in iteration k (so beta[m_eff-1] is the final
    residual norm, not an entry of T)."""
    q = np.asarray(q0, dtype=np.float64)
    q = q / np.linalg.norm(q)
    q_prev = None
    alpha, beta = [], []
    Q = [q.copy()]
    for k in range(m):
        r = np.asarray(apply_H(q), dtype=np.float64).copy()
        if k > 0:
            r -= beta[k - 1] * q_prev
        a = float(q @ r)
        r -= a * q
        if reorth == "full":
            Qm = np.stack(Q)                      # q_0 .. q_k
            before = np.linalg.norm(r)
            c = Qm @ r
            r -= Qm.T @ c
            if np.linalg.norm(r) < before / np.sqrt(2.0):
                c = Qm @ r
                r -= Qm.T @ c
        b = float(np.linalg.norm(r))
        alpha.append(a)
        beta.append(b)
        if b < tol:
            break
        q_prev, q = q, r / b
        Q.append(q.copy())
    m_eff = len(alpha)
    out = (np.array(alpha), np.array(beta), m_eff)
    if return_basis:
        out = out + (np.stack(Q),)
    return out


def tridiagonal(alpha, beta):
    """T_k: alpha on the diagonal, beta_0..beta_{k-2} beside it."""
    k = len(alpha)
    T = np.diag(np.asarray(alpha, dtype=np.float64))
    for i in range(k - 1):
        T[i, i + 1] = T[i + 1, i] = beta[i]
    return T


def slq_readout(alpha, beta):
    """(ritz ascending, weights) with weights_i = (first component of the i-th
    unit eigenvector of T_k)^2."""
    theta, Y = np.linalg.eigh(tridiagonal(alpha, beta))
    return theta, Y[0, :] ** 2


def slq(apply_H, probes, m, reorth="none", tol=0.0):
    """Per-probe (alpha, beta, ritz, weights, m_eff); no averaging over probes."""
    res = []
    for z in probes:
        a, b, m_eff = lanczos(apply_H, z, m, reorth, tol)
        th, w = slq_readout(a, b)
        res.append((a, b, th, w, m_eff))
    return res
