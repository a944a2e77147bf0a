"""Pins of the CPU oracle against things other than itself (no GPU needed).

The oracle follows the element-wise MTTKRP definition (paper Sec. II-B,
Eq. (elem), lambda = 1).  Each test here would fail for a plausible mistake in
it: a dropped factor, a wrong mode skipped, a transposed factor, a wrong
stride, a wrong output row.
"""
import itertools
import os

import numpy as np
import pytest

from paper_2510_14891_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_problem(dims, R, seed, dtype=np.float64, lo=-1.0, hi=1.0):
    """Seeded X (logical ndarray, Fortran order) and factors."""
    import torch
    tdt = torch.float64 if dtype == np.float64 else torch.float32
    N = int(np.prod(dims))
    flat = inputs.uniform(seed, N, lo, hi, dtype=tdt)
    X = inputs.as_ndarray_view(flat, dims)
    A = [inputs.uniform(seed + 100 + m, (I, R), lo, hi, dtype=tdt).numpy()
         for m, I in enumerate(dims)]
    return X, A


# ---------------------------------------------------------------- P1 brute force
def unfold_naive(X, k):
    """Mode-k matricization by the column formula of Sec. II-A (0-based):
    col = sum_{l != k} i_l * prod_{m < l, m != k} I_m."""
    dims = X.shape
    d = len(dims)
    ncol = int(np.prod(dims)) // dims[k]
    Xk = np.zeros((dims[k], ncol))
    for idx in itertools.product(*[range(I) for I in dims]):
        col, mult = 0, 1
        for l in range(d):
            if l == k:
                continue
            col += idx[l] * mult
            mult *= dims[l]
        Xk[idx[k], col] = X[idx]
    return Xk


def khatri_rao_naive(Amat, Bmat):
    """Column-wise Kronecker product (Sec. II-A): column j is a_j (x) b_j."""
    m, p = Amat.shape
    n, p2 = Bmat.shape
    assert p == p2
    out = np.zeros((m * n, p))
    for j in range(p):
        for a in range(m):
            for b in range(n):
                out[a * n + b, j] = Amat[a, j] * Bmat[b, j]
    return out


def mttkrp_matrix_based(X, A, k):
    """Eq. (krp): G = X_(k) Z with Z = A_d (.) ... (.) A_{k+1} (.) A_{k-1} (.) ... (.) A_1."""
    d = X.ndim
    modes = [m for m in range(d - 1, -1, -1) if m != k]   # d, ..., 1 skipping k
    Z = A[modes[0]]
    for m in modes[1:]:
        Z = khatri_rao_naive(Z, A[m])
    Xk = unfold_naive(X, k)
    M = np.zeros((X.shape[k], Z.shape[1]))
    for n in range(Xk.shape[0]):
        for j in range(Z.shape[1]):
            s = 0.0
            for c in range(Xk.shape[1]):
                s += Xk[n, c] * Z[c, j]
            M[n, j] = s
    return M


@pytest.mark.parametrize("dims,R", [
    ((2, 3, 4), 3), ((3, 1, 2, 2), 1), ((2, 2, 2, 2, 3), 3), ((7, 5, 3), 3),
    ((4, 3), 2), ((1, 5, 1), 2), ((3, 2, 2, 2, 2, 2), 2),
])
def test_p1_matches_explicit_unfold_times_explicit_krp(oracle, dims, R):
    X, A = rand_problem(dims, R, seed=11)
    for k in range(len(dims)):
        ref = mttkrp_matrix_based(X, A, k)
        got = oracle.mttkrp(X, A, k)
        assert got.shape == (dims[k], R)
        assert oracle.normwise_rel_err(got, ref) <= 1e-14, (dims, k)
        # the natively accumulated build is the same sum, same order
        got_n = oracle.mttkrp(X, A, k, native_acc=True)
        assert oracle.normwise_rel_err(got_n, ref) <= 1e-13


# ---------------------------------------------------------------- hand-worked golden
def read_worked():
    vals = {}
    with open(os.path.join(GOLDEN, "worked_2x2x2.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            vals[parts[0]] = np.array([float(v) for v in parts[1:]])
    return vals


def test_hand_worked_example(oracle):
    v = read_worked()
    X = np.reshape(v["X"], (2, 2, 2), order="F")
    A = [v["A%d" % m].reshape(2, 2) for m in range(3)]
    for k in range(3):
        got = oracle.mttkrp(X, A, k)
        assert np.array_equal(got, v["M%d" % k].reshape(2, 2)), k
        got32 = oracle.mttkrp(X.astype(np.float32), [a.astype(np.float32) for a in A], k)
        assert np.array_equal(got32, v["M%d" % k].reshape(2, 2).astype(np.float32))


# ---------------------------------------------------------------- P2 / P3 closed forms
@pytest.mark.parametrize("dims", [(9, 7, 5), (6, 5, 4, 3), (3, 4, 2, 5, 3)])
def test_p2_rank1_closed_form(oracle, dims):
    """X = a_0 o a_1 o ... => M(:, r) = a_k * prod_{m != k} (a_m^T A_m(:, r))."""
    import torch
    R = 4
    vecs = [inputs.normal(500 + m, I).numpy() for m, I in enumerate(dims)]
    X = vecs[0]
    for v in vecs[1:]:
        X = np.multiply.outer(X, v)
    _, A = rand_problem(dims, R, seed=21)
    for k in range(len(dims)):
        scale = np.ones(R)
        for m in range(len(dims)):
            if m != k:
                scale = scale * (vecs[m] @ A[m])
        ref = np.outer(vecs[k], scale)
        got = oracle.mttkrp(X, A, k)
        assert oracle.normwise_rel_err(got, ref) <= 1e-13


@pytest.mark.parametrize("dims,S", [((8, 6, 7), 3), ((5, 4, 6, 3), 5)])
def test_p3_kruskal_closed_form(oracle, dims, S):
    """X = [[U_0..U_{d-1}]] => M = U_k (hadamard_{m != k} U_m^T A_m)."""
    R = 6
    U = [inputs.normal(600 + m, (I, S)).numpy() for m, I in enumerate(dims)]
    X = np.zeros(dims)
    for s in range(S):
        t = U[0][:, s]
        for m in range(1, len(dims)):
            t = np.multiply.outer(t, U[m][:, s])
        X += t
    _, A = rand_problem(dims, R, seed=31)
    for k in range(len(dims)):
        H = np.ones((S, R))
        for m in range(len(dims)):
            if m != k:
                H = H * (U[m].T @ A[m])
        ref = U[k] @ H
        assert oracle.normwise_rel_err(oracle.mttkrp(X, A, k), ref) <= 1e-13
    # CP-ALS identity: with U = A, M = A_k hadamard_{m != k}(A_m^T A_m)
    Xa = np.zeros(dims)
    for s in range(R):
        t = A[0][:, s]
        for m in range(1, len(dims)):
            t = np.multiply.outer(t, A[m][:, s])
        Xa += t
    for k in range(len(dims)):
        H = np.ones((R, R))
        for m in range(len(dims)):
            if m != k:
                H = H * (A[m].T @ A[m])
        assert oracle.normwise_rel_err(oracle.mttkrp(Xa, A, k), A[k] @ H) <= 1e-13


# ---------------------------------------------------------------- P4 linearity
def test_p4_linearity(oracle):
    dims, R = (6, 5, 4, 3), 5
    X, A = rand_problem(dims, R, seed=41)
    Y, B = rand_problem(dims, R, seed=42)
    al, be = 0.75, -2.5
    for k in range(4):
        lhs = oracle.mttkrp(al * X + be * Y, A, k)
        rhs = al * oracle.mttkrp(X, A, k) + be * oracle.mttkrp(Y, A, k)
        assert oracle.normwise_rel_err(lhs, rhs) <= 1e-14
        # linear in each factor m != k
        m = (k + 1) % 4
        A2 = list(A)
        A2[m] = al * A[m] + be * B[m]
        Ab = list(A)
        Ab[m] = B[m]
        lhs = oracle.mttkrp(X, A2, k)
        rhs = al * oracle.mttkrp(X, A, k) + be * oracle.mttkrp(X, Ab, k)
        assert oracle.normwise_rel_err(lhs, rhs) <= 1e-14
        # scaling the columns of a factor scales the columns of M
        s = np.arange(1, R + 1, dtype=np.float64)
        A3 = list(A)
        A3[m] = A[m] * s
        assert oracle.normwise_rel_err(oracle.mttkrp(X, A3, k),
                                       oracle.mttkrp(X, A, k) * s) <= 1e-14


# ---------------------------------------------------------------- P5 independence
def test_p5_independent_of_Ak_and_of_other_subtensors(oracle):
    dims, R = (5, 4, 6), 3
    X, A = rand_problem(dims, R, seed=51)
    for k in range(3):
        base = oracle.mttkrp(X, A, k)
        A_nan = list(A)
        A_nan[k] = np.full_like(A[k], np.nan)
        assert np.array_equal(oracle.mttkrp(X, A_nan, k), base)
        A_none = list(A)
        A_none[k] = None
        assert np.array_equal(oracle.mttkrp(X, A_none, k), base)
        # row n depends only on the mode-k subtensor n (Sec. III)
        n = 2
        Y = X.copy(order="F")
        sl = [slice(None)] * 3
        sl[k] = n
        keep = Y[tuple(sl)].copy()
        Y[...] = 123.0
        Y[tuple(sl)] = keep
        assert np.array_equal(oracle.mttkrp(Y, A, k)[n], base[n])
        # and the row request returns exactly those rows
        rows = [n, 0, dims[k] - 1, n]
        assert np.array_equal(oracle.mttkrp(X, A, k, rows=rows), base[rows])


# ---------------------------------------------------------------- P6 marginals
def test_p6_marginals(oracle):
    dims, R = (4, 6, 5, 3), 4
    X, A = rand_problem(dims, R, seed=61)
    ones = [np.ones_like(a) for a in A]
    for k in range(4):
        axes = tuple(m for m in range(4) if m != k)
        ref = np.repeat(X.sum(axis=axes)[:, None], R, axis=1)
        assert oracle.normwise_rel_err(oracle.mttkrp(X, ones, k), ref) <= 1e-14
        colprod = np.ones(R)
        for m in range(4):
            if m != k:
                colprod = colprod * A[m].sum(axis=0)
        ref = np.repeat(colprod[None, :], dims[k], axis=0)
        assert oracle.normwise_rel_err(oracle.mttkrp(np.ones(dims), A, k), ref) <= 1e-13


# ---------------------------------------------------------------- P7 library special cases
def test_p7_matrix_case_is_matmul(oracle):
    X, A = rand_problem((13, 9), 5, seed=71)
    assert oracle.normwise_rel_err(oracle.mttkrp(X, A, 0), X @ A[1]) <= 1e-14
    assert oracle.normwise_rel_err(oracle.mttkrp(X, A, 1), X.T @ A[0]) <= 1e-14


def test_p7_einsum(oracle):
    X, A = rand_problem((7, 6, 5), 4, seed=72)
    assert oracle.normwise_rel_err(
        oracle.mttkrp(X, A, 0), np.einsum("abc,br,cr->ar", X, A[1], A[2])) <= 1e-14
    assert oracle.normwise_rel_err(
        oracle.mttkrp(X, A, 1), np.einsum("abc,ar,cr->br", X, A[0], A[2])) <= 1e-14
    assert oracle.normwise_rel_err(
        oracle.mttkrp(X, A, 2), np.einsum("abc,ar,br->cr", X, A[0], A[1])) <= 1e-14
    X4, A4 = rand_problem((3, 4, 5, 2), 3, seed=73)
    assert oracle.normwise_rel_err(
        oracle.mttkrp(X4, A4, 2),
        np.einsum("abcd,ar,br,dr->cr", X4, A4[0], A4[1], A4[3])) <= 1e-14
    # float32 data, long-double accumulation: exact products of fp32 inputs
    X32, A32 = rand_problem((7, 6, 5), 4, seed=74, dtype=np.float32)
    ref = np.einsum("abc,br,cr->ar", X32.astype(np.float64),
                    A32[1].astype(np.float64), A32[2].astype(np.float64))
    got = oracle.mttkrp(X32, A32, 0)
    assert got.dtype == np.float32
    assert oracle.normwise_rel_err(got, ref) <= 1e-7


# ---------------------------------------------------------------- P8 permutation equivariance
def test_p8_mode_permutation(oracle):
    dims, R = (4, 5, 3, 6), 3
    X, A = rand_problem(dims, R, seed=81)
    for perm in [(1, 0, 2, 3), (3, 2, 1, 0), (2, 3, 0, 1)]:
        Xp = np.asfortranarray(np.transpose(X, perm))
        Ap = [A[p] for p in perm]
        for knew, kold in enumerate(perm):
            a = oracle.mttkrp(Xp, Ap, knew)
            b = oracle.mttkrp(X, A, kold)
            assert oracle.normwise_rel_err(a, b) <= 1e-14


# ---------------------------------------------------------------- P10 error bound
def test_p10_long_double_vs_native_within_bound(oracle):
    """Plain double accumulation of N_S terms differs from the long-double sum
    by at most about 8 u sqrt(N_S) normwise on random data, and the long-double
    build really is more accurate than the native one (exact rational check)."""
    assert oracle.long_double_mant_bits() >= 64
    dims, R = (40, 30, 20), 4
    X, A = rand_problem(dims, R, seed=91, lo=0.0, hi=1.0)
    u = 2.0 ** -53
    for k in range(3):
        NS = np.prod(dims) / dims[k]
        hi = oracle.mttkrp(X, A, k)
        lo = oracle.mttkrp(X, A, k, native_acc=True)
        assert oracle.normwise_rel_err(lo, hi) <= 8 * u * np.sqrt(NS)
    # exact check on a tiny case with Python fractions
    from fractions import Fraction
    dims, R = (3, 4, 3), 2
    X, A = rand_problem(dims, R, seed=92)
    k = 1
    exact = np.zeros((dims[k], R))
    for n in range(dims[k]):
        for j in range(R):
            s = Fraction(0)
            for i0 in range(dims[0]):
                for i2 in range(dims[2]):
                    s += (Fraction(float(X[i0, n, i2])) * Fraction(float(A[0][i0, j]))
                          * Fraction(float(A[2][i2, j])))
            exact[n, j] = float(s)
    got = oracle.mttkrp(X, A, k)
    assert np.max(np.abs(got - exact)) <= 2.0 ** -52 * np.max(np.abs(exact))


def test_bad_arguments_rejected(oracle):
    X, A = rand_problem((3, 4, 5), 2, seed=95)
    with pytest.raises(Exception):
        oracle.mttkrp(X, A, 3)
    with pytest.raises(Exception):
        oracle.mttkrp(X, A, 0, rows=[3])
    with pytest.raises(Exception):
        oracle.mttkrp(X, [A[0], None, A[2]], 0)


# ---------------------------------------------------------------- input generator
def test_generator_is_index_addressed_and_matches_scalar_hash():
    import torch
    z = inputs.hash_bits(1234, 0, 50)
    for i in (0, 1, 7, 49):
        want = inputs.hash_bits_scalar(1234, i)
        got = int(z[i].item()) & ((1 << 64) - 1)
        assert got == want
    a = inputs.uniform(7, 1000)
    b = torch.empty(300, dtype=torch.float64)
    inputs.fill_uniform(b, 7, offset=500)
    assert torch.equal(a[500:800], b)
    assert 0.0 <= float(a.min()) and float(a.max()) < 1.0
    g = inputs.normal(9, 200000)
    assert abs(float(g.mean())) < 0.01 and abs(float(g.std()) - 1.0) < 0.01
    g2 = torch.empty(100, dtype=torch.float64)
    inputs.fill_normal(g2, 9, offset=1000)
    assert torch.equal(g[1000:1100], g2)


def test_cp_noise_recipe_small():
    import torch
    w = inputs.scaled(inputs.WORKLOADS["c4_48x48x48x48x48_f32_R64"], (6, 5, 4, 3, 4))
    flat = inputs.make_tensor(w)
    assert flat.dtype == torch.float32 and flat.numel() == 6 * 5 * 4 * 3 * 4
    # noise level: X - X_cp has rms = 1 % of rms(X_cp)
    S = 8
    U = [inputs.normal(3000 + m, (I, S)).numpy() for m, I in enumerate(w.dims)]
    Xcp = np.zeros(w.dims)
    for s in range(S):
        t = U[0][:, s]
        for m in range(1, 5):
            t = np.multiply.outer(t, U[m][:, s])
        Xcp += t
    X = inputs.as_ndarray_view(flat, w.dims).astype(np.float64)
    rms = np.sqrt(np.mean(Xcp ** 2))
    ratio = np.sqrt(np.mean((X - Xcp) ** 2)) / rms
    assert 0.005 < ratio < 0.02


# ---------------------------------------------------------------- weight vector lambda
def test_lambda_is_a_column_scaling(oracle):
    """Eq. (krp): G = Y_(k) Z diag(lambda); Eq. (elem): the factor lambda_j."""
    dims, R, S = (6, 5, 4), 4, 3
    X, A = rand_problem(dims, R, seed=97)
    lam = np.array([0.5, -2.0, 3.0, 1.25])
    for k in range(3):
        base = oracle.mttkrp(X, A, k)
        assert np.array_equal(oracle.mttkrp(X, A, k, lam=np.ones(R)), base)
        assert oracle.normwise_rel_err(oracle.mttkrp(X, A, k, lam=lam), base * lam) <= 1e-15
        # against the matrix-based definition with the explicit diag(lambda)
        ref = mttkrp_matrix_based(X, A, k) @ np.diag(lam)
        assert oracle.normwise_rel_err(oracle.mttkrp(X, A, k, lam=lam), ref) <= 1e-14
    # closed form: X = [[mu; U_0, U_1, U_2]]  =>  M = U_k diag(mu) (hadamard U_m^T A_m) diag(lambda)
    U = [inputs.normal(700 + m, (I, S)).numpy() for m, I in enumerate(dims)]
    mu = np.array([2.0, 0.5, -1.0])
    Xk = np.zeros(dims)
    for s in range(S):
        t = mu[s] * U[0][:, s]
        for m in range(1, 3):
            t = np.multiply.outer(t, U[m][:, s])
        Xk += t
    for k in range(3):
        H = np.ones((S, R))
        for m in range(3):
            if m != k:
                H = H * (U[m].T @ A[m])
        ref = (U[k] * mu) @ H * lam
        assert oracle.normwise_rel_err(oracle.mttkrp(Xk, A, k, lam=lam), ref) <= 1e-13


# ---------------------------------------------------------------- tile-volume heuristic
def _heuristic_cases():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_tile_heuristic.txt")
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [t.strip() for t in line.split("|")]
        yield f[0], [int(t) for t in f[1].split()], int(f[2]), int(f[3]), int(f[4]), int(f[5]), int(f[6])


def test_tile_heuristic_matches_the_papers_values():
    """Eq. (heuristic) against the tile sizes the paper reports (Sec. IV-C)."""
    from oracle import tile_heuristic
    n = 0
    for label, dims, cache, vb, c, width, vol in _heuristic_cases():
        assert tile_heuristic.tile_volume(dims, cache, vb, c) == (width, vol), label
        n += 1
    assert n == 4


def test_tile_heuristic_properties():
    """The width is the integer (d-1)-th root of the budget, capped by the smallest extent."""
    from oracle import tile_heuristic
    import math
    for d in (2, 3, 4, 5, 6):
        for cache in (16384, 32768, 65536, 262144, 1 << 21):
            for vb in (4, 8):
                for c in (1, 2, 8, 64):
                    dims = [10 ** 9] * d
                    w, vol = tile_heuristic.tile_volume(dims, cache, vb, c)
                    budget = cache / 4 / (vb * c / 2)
                    assert vol == w ** (d - 1)
                    assert w == 1 or w ** (d - 1) <= budget
                    assert (w + 1) ** (d - 1) > budget
                    assert abs(w - math.floor(budget ** (1.0 / (d - 1)) + 1e-9)) <= 1
                    # cap by the smallest extent
                    w2, vol2 = tile_heuristic.tile_volume([10 ** 9] * (d - 1) + [3], cache, vb, c)
                    assert w2 == min(w, 3) and vol2 == w2 ** (d - 1)
