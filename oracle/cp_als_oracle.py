"""Oracle of the CP-ALS driver built on the MTTKRP (paper Sec. I and Sec. IV-C:
the MTTKRP is the bottleneck kernel of CP-ALS; the paper runs CP-ALS "with
tolerance 1e-4" and names its other operations only as "inner-product,
Cholesky solve, etc.").

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/`` may import this
module.  Plain numpy in fp64; the MTTKRP step calls the definition oracle
(``mttkrp_oracle``), the linear algebra steps call numpy's library routines.
Nothing here imports the HIP package.

The paper does not print the iteration; this is the textbook alternating least
squares for the CP model of Sec. II-A (X ~ sum_j lambda_j a_j^(1) o ... o a_j^(d)),
in the order stated below, which the GPU driver follows too:

  for every sweep, for k = 0 .. d-1:
      M   = MTTKRP(X, {A_m}, k)                          Eq. (elem), lambda = 1
      V   = Hadamard product of the Gram matrices A_m^T A_m, m != k
      A_k = M V^{-1}                                      (V = L L^T, two triangular solves)
      lambda_j = || A_k(:, j) ||_2 ;  A_k(:, j) /= lambda_j   (columns of norm 0 are left alone, lambda_j = 0)
  after the last mode of a sweep:
      <X, X^>  = sum_j lambda_j sum_i M(i, j) A_{d-1}(i, j)
      ||X^||^2 = lambda^T (Hadamard product of all d Gram matrices) lambda
      fit      = 1 - sqrt(max(||X||^2 + ||X^||^2 - 2 <X, X^>, 0)) / ||X||
  stop when |fit - previous fit| < tol or after max_iters sweeps.
"""
from typing import List, Sequence, Tuple

import numpy as np

from oracle import mttkrp_oracle


def cp_als(X: np.ndarray, factors: Sequence[np.ndarray], max_iters: int, tol: float
           ) -> Tuple[List[np.ndarray], np.ndarray, List[float]]:
    """X: ndarray of shape dims (logical indexing).  factors: initial A_m (I_m x R).
    Returns (factors, lambda, fit after every sweep)."""
    d = X.ndim
    A = [np.array(a, dtype=np.float64, copy=True) for a in factors]
    R = A[0].shape[1]
    X = np.asarray(X, dtype=np.float64)
    normX = float(np.sqrt(np.sum(X.astype(np.longdouble) ** 2)))
    G = [a.T @ a for a in A]
    lam = np.ones(R)
    fits: List[float] = []
    for _ in range(max_iters):
        M = None
        for k in range(d):
            M = mttkrp_oracle.mttkrp(X, A, k)
            V = np.ones((R, R))
            for m in range(d):
                if m != k:
                    V = V * G[m]
            L = np.linalg.cholesky(V)
            # A_k = M V^{-1}:  solve L y = M^T, then L^T z = y
            Y = np.linalg.solve(L, M.T)
            Z = np.linalg.solve(L.T, Y)
            Ak = Z.T
            lam = np.sqrt(np.sum(Ak * Ak, axis=0))
            scale = np.where(lam > 0, lam, 1.0)
            A[k] = Ak / scale
            G[k] = A[k].T @ A[k]
        iprod = float(np.sum(lam * np.sum(M * A[d - 1], axis=0)))
        Vall = np.ones((R, R))
        for m in range(d):
            Vall = Vall * G[m]
        norm_model2 = float(lam @ Vall @ lam)
        resid2 = max(normX * normX + norm_model2 - 2.0 * iprod, 0.0)
        fit = 1.0 - np.sqrt(resid2) / normX
        fits.append(fit)
        if len(fits) > 1 and abs(fits[-1] - fits[-2]) < tol:
            break
    return A, lam, fits


def reconstruct(factors: Sequence[np.ndarray], lam: np.ndarray) -> np.ndarray:
    """Full tensor of the model, for small shapes (brute force)."""
    d = len(factors)
    dims = [a.shape[0] for a in factors]
    R = factors[0].shape[1]
    out = np.zeros(dims)
    for j in range(R):
        t = lam[j]
        for m in range(d):
            shape = [1] * d
            shape[m] = dims[m]
            t = t * factors[m][:, j].reshape(shape)
        out = out + t
    return out
