"""Pins of the CP-ALS oracle (oracle/cp_als_oracle.py) against what the
mathematics fixes, independent of the oracle's own formulas:

* one mode update is the least-squares solution of min ||X_(k) - A Z^T||_F, checked
  with numpy.linalg.lstsq on an explicitly unfolded X and an explicitly formed
  Khatri-Rao matrix (Sec. II-A definitions);
* the fit it reports equals 1 - ||X - X^||_F / ||X||_F with X^ rebuilt entry by entry;
* the fit never decreases from sweep to sweep (each update minimises the residual);
* an exactly rank-R tensor is recovered (fit -> 1).
"""
import numpy as np

from oracle import cp_als_oracle


def unfold(X, k):
    """X_(k): rows = mode k, columns with the first remaining index fastest."""
    d = X.ndim
    order = [k] + [m for m in range(d) if m != k]
    return np.transpose(X, order).reshape(X.shape[k], -1, order="F")


def khatri_rao_excluding(A, k):
    """Rows indexed like the columns of X_(k): first remaining mode fastest."""
    mats = [A[m] for m in range(len(A)) if m != k]
    R = mats[0].shape[1]
    Z = np.ones((1, R))
    for a in mats:                     # later modes vary slower
        Z = (a[:, None, :] * Z[None, :, :]).reshape(-1, R)
    return Z


def rng_problem(dims, R, seed, rank_true=None, noise=0.0):
    rng = np.random.default_rng(seed)
    if rank_true is None:
        X = rng.standard_normal(dims)
    else:
        U = [rng.standard_normal((I, rank_true)) for I in dims]
        X = cp_als_oracle.reconstruct(U, np.ones(rank_true))
        X = X + noise * rng.standard_normal(dims)
    A0 = [rng.standard_normal((I, R)) for I in dims]
    return X, A0


def test_one_update_is_the_least_squares_solution():
    dims, R = (6, 5, 4), 3
    X, A0 = rng_problem(dims, R, 1)
    # run one sweep by hand around the oracle: after the update of mode 0, A_0 * diag(lambda)
    # must solve the least-squares problem with the *initial* other factors
    A, lam, fits = cp_als_oracle.cp_als(X, A0, 1, 0.0)
    # replay: mode 0 update used A0[1], A0[2]
    Z = khatri_rao_excluding(A0, 0)
    sol, *_ = np.linalg.lstsq(Z, unfold(X, 0).T, rcond=None)
    # the sweep then went on to modes 1 and 2 with the normalised A_0; redo mode 0 alone to compare
    A1, lam1, _ = _single_mode_update(X, A0, 0)
    np.testing.assert_allclose(A1 * lam1, sol.T, rtol=1e-9, atol=1e-11)


def _single_mode_update(X, A0, k):
    """Mode-k update by the independent route (lstsq), normalised like the oracle."""
    Z = khatri_rao_excluding(A0, k)
    sol, *_ = np.linalg.lstsq(Z, unfold(X, k).T, rcond=None)
    Ak = sol.T
    lam = np.linalg.norm(Ak, axis=0)
    return Ak / lam, lam, None


def test_sweep_matches_independent_least_squares_chain():
    """A full sweep redone with lstsq updates (no Gram matrices, no Cholesky, no MTTKRP)."""
    for dims, R, seed in (((6, 5, 4), 3, 2), ((4, 3, 5, 2), 2, 3), ((7, 6), 2, 4)):
        X, A0 = rng_problem(dims, R, seed)
        A, lam, fits = cp_als_oracle.cp_als(X, A0, 1, 0.0)
        B = [a.copy() for a in A0]
        lam_b = None
        for k in range(len(dims)):
            B[k], lam_b, _ = _single_mode_update(X, B, k)
        for m in range(len(dims)):
            np.testing.assert_allclose(A[m], B[m], rtol=1e-8, atol=1e-10)
        np.testing.assert_allclose(lam, lam_b, rtol=1e-8)


def test_fit_equals_brute_force_residual():
    for dims, R, seed in (((6, 5, 4), 3, 5), ((3, 4, 2, 3), 2, 6)):
        X, A0 = rng_problem(dims, R, seed)
        A, lam, fits = cp_als_oracle.cp_als(X, A0, 4, 0.0)
        Xh = cp_als_oracle.reconstruct(A, lam)
        fit = 1.0 - np.linalg.norm(X - Xh) / np.linalg.norm(X)
        assert abs(fit - fits[-1]) < 1e-10
        assert len(fits) == 4


def test_fit_is_monotone_and_tolerance_stops():
    X, A0 = rng_problem((8, 7, 6), 4, 7, rank_true=4, noise=0.05)
    _, _, full = cp_als_oracle.cp_als(X, A0, 60, 0.0)
    assert len(full) == 60
    assert all(b >= a - 1e-12 for a, b in zip(full, full[1:]))
    for tol in (1e-2, 2.6e-3, 1e-4):
        _, _, fits = cp_als_oracle.cp_als(X, A0, 60, tol)
        first = next((i for i in range(1, 60) if abs(full[i] - full[i - 1]) < tol), 59)
        assert len(fits) == first + 1, (tol, len(fits), first)
        np.testing.assert_allclose(fits, full[:first + 1], rtol=0, atol=0)


def test_exact_low_rank_tensor_is_recovered():
    X, A0 = rng_problem((9, 8, 7), 2, 8, rank_true=2)
    A, lam, fits = cp_als_oracle.cp_als(X, A0, 200, 1e-13)
    assert fits[-1] > 1.0 - 1e-6
    for a in A:
        np.testing.assert_allclose(np.linalg.norm(a, axis=0), 1.0, rtol=1e-12)
