"""Pins of the two error measures every parity assertion goes through
(``normwise_rel_err`` and ``rowwise_rel_err`` of the oracle's front end), and a
mutation check of the gate itself.  No GPU needed.

The parity criterion is the normwise relative error ||M - M_ref||_F / ||M_ref||_F
<= 1e-12 (fp64) / 1e-5 (fp32) between results of Eq. (elem) (paper Sec. II-B).
The values below are worked out by hand, so a comparator that dropped a square
root, squared the ratio, normalised by the wrong operand or summed absolute
values instead of squares fails one of them.
"""
import numpy as np
import pytest

from paper_2510_14891_amd import inputs

TOL64 = 1e-12
TOL32 = 1e-5


def test_normwise_hand_computed_ratio(oracle):
    # ||ref||_F = sqrt(9 + 16) = 5; the difference has one entry d, so the error is d / 5
    ref = np.array([[3.0, 4.0], [0.0, 0.0]])
    for d, want in ((1e-11, 2e-12), (1e-12, 2e-13), (5.0, 1.0), (0.5, 0.1)):
        test = ref + np.array([[0.0, 0.0], [0.0, d]])
        got = oracle.normwise_rel_err(test, ref)
        assert got == pytest.approx(want, rel=1e-12), (d, got)
    # the first is above the fp64 gate, the second below it
    assert oracle.normwise_rel_err(ref + np.array([[0, 0], [0, 1e-11]]), ref) > TOL64
    assert oracle.normwise_rel_err(ref + np.array([[0, 0], [0, 1e-12]]), ref) <= TOL64


def test_normwise_is_a_two_norm_not_a_one_norm_or_a_square(oracle):
    # difference (1, 1, 1, 1) against reference (2, 2, 2, 2): sqrt(4) / sqrt(16) = 1/2
    # (sum of absolute values would give 4/8 = 1/2 as well, so take an uneven one too)
    ref = np.full((2, 2), 2.0)
    assert oracle.normwise_rel_err(ref + 1.0, ref) == pytest.approx(0.5, rel=1e-15)
    # difference (3, 4) against reference (6, 8): 5 / 10; a 1-norm gives 7/14, a squared ratio 1/4,
    # a max-norm 4/8; difference (1, 0) against (3, 4): 1/5; 1-norm 1/7, squared 1/25, max 1/4
    assert oracle.normwise_rel_err(np.array([[9.0, 12.0]]), np.array([[6.0, 8.0]])) == pytest.approx(0.5, rel=1e-15)
    assert oracle.normwise_rel_err(np.array([[4.0, 4.0]]), np.array([[3.0, 4.0]])) == pytest.approx(0.2, rel=1e-15)
    # not symmetric: the reference normalises
    assert oracle.normwise_rel_err(np.array([[3.0, 4.0]]), np.array([[4.0, 4.0]])) == pytest.approx(
        1.0 / np.sqrt(32.0), rel=1e-15)


def test_normwise_sign_and_scale(oracle):
    ref = np.array([[1.0, -2.0, 2.0]])          # norm 3
    assert oracle.normwise_rel_err(-ref, ref) == pytest.approx(2.0, rel=1e-15)
    assert oracle.normwise_rel_err(ref, ref) == 0.0
    assert oracle.normwise_rel_err(1e150 * (ref + [[0, 0, 3e-6]]), 1e150 * ref) == pytest.approx(1e-6, rel=1e-9)
    # fp32 inputs are promoted, not compared in fp32
    a = np.array([[1.0, 1.0]], dtype=np.float32)
    b = np.array([[1.0, 1.0 + 2.0 ** -23]], dtype=np.float32)
    assert oracle.normwise_rel_err(a, b) == pytest.approx(2.0 ** -23 / np.sqrt(1.0 + (1.0 + 2.0 ** -23) ** 2), rel=1e-12)


def test_normwise_zero_reference_and_nan(oracle):
    z = np.zeros((3, 2))
    assert oracle.normwise_rel_err(z, z) == 0.0
    assert oracle.normwise_rel_err(z + 1e-300, z) == float("inf")
    bad = np.array([[np.nan, 1.0]])
    assert not oracle.normwise_rel_err(bad, np.array([[1.0, 1.0]])) <= TOL64   # NaN never passes a "<= tol" gate
    assert not oracle.normwise_rel_err(np.array([[np.inf, 1.0]]), np.array([[1.0, 1.0]])) <= TOL64


def test_normwise_shape_mismatch_raises(oracle):
    with pytest.raises(ValueError):
        oracle.normwise_rel_err(np.zeros((2, 3)), np.zeros((3, 2)))
    with pytest.raises(ValueError):
        oracle.normwise_rel_err(np.zeros((2, 3)), np.zeros((2, 4)))


def test_rowwise_hand_computed(oracle):
    # rows of norm 5 and 1e-6: an error of 1e-9 in the small row is 2e-10 of the whole
    # matrix (passes a 1e-9 normwise gate) but 1e-3 of its own row
    ref = np.array([[3.0, 4.0], [1e-6, 0.0]])
    test = ref + np.array([[0.0, 0.0], [0.0, 1e-9]])
    assert oracle.normwise_rel_err(test, ref) == pytest.approx(2e-10, rel=1e-6)
    assert oracle.rowwise_rel_err(test, ref) == pytest.approx(1e-3, rel=1e-12)
    # the worst row counts, wherever it is
    test2 = ref + np.array([[0.0, 0.5], [0.0, 0.0]])
    assert oracle.rowwise_rel_err(test2, ref) == pytest.approx(0.1, rel=1e-12)
    assert oracle.rowwise_rel_err(ref, ref) == 0.0
    # a zero reference row must be zero in the result
    refz = np.array([[1.0, 0.0], [0.0, 0.0]])
    assert oracle.rowwise_rel_err(refz, refz) == 0.0
    assert oracle.rowwise_rel_err(refz + np.array([[0.0, 0.0], [1e-300, 0.0]]), refz) == float("inf")
    nan = refz.copy()
    nan[0, 1] = np.nan
    assert not oracle.rowwise_rel_err(nan, refz) <= 1.0
    with pytest.raises(ValueError):
        oracle.rowwise_rel_err(np.zeros((2, 3)), np.zeros((3, 2)))
    with pytest.raises(ValueError):
        oracle.rowwise_rel_err(np.zeros(3), np.zeros(3))


# ---------------------------------------------------------------- mutation check of the gate
def _einsum_mttkrp(X, A, k, mutate=None):
    """Eq. (elem) for d = 3 by numpy.einsum (independent of the oracle's C loop), with an
    optional planted mistake."""
    letters = "abc"
    ops = [A[m] for m in range(3) if m != k]
    subs = [letters[m] + "r" for m in range(3) if m != k]
    if mutate == "dropped_factor":
        ops, subs = ops[:1], subs[:1]
    elif mutate == "swapped_factors":            # needs equal extents of the two modes
        ops = ops[::-1]
    elif mutate == "reversed_factor_rows":       # transposed index: row I-1-i instead of i
        ops = [ops[0][::-1]] + ops[1:]
    M = np.einsum("abc," + ",".join(subs) + "->" + letters[k] + "r", X, *ops)
    if mutate == "shifted_output_row":
        M = np.roll(M, 1, axis=0)
    elif mutate == "one_entry_missing":          # one tensor entry left out of one sum
        others = [m for m in range(3) if m != k]
        idx = [1, 1, 1]
        M = M.copy()
        M[idx[k]] -= X[1, 1, 1] * A[others[0]][idx[others[0]]] * A[others[1]][idx[others[1]]]
    elif mutate == "fp32_accumulation":          # the sums taken in single precision
        M = np.einsum("abc," + ",".join(subs) + "->" + letters[k] + "r", X.astype(np.float32),
                      *[o.astype(np.float32) for o in ops]).astype(np.float64)
    return M


@pytest.mark.parametrize("mutate", ["dropped_factor", "swapped_factors", "reversed_factor_rows",
                                    "shifted_output_row", "one_entry_missing", "fp32_accumulation"])
def test_gate_rejects_planted_mistakes(oracle, mutate):
    """The gate the GPU parity tests use (normwise error of a result against the oracle,
    <= 1e-12) accepts the correct result and rejects each planted mistake."""
    import torch
    dims, R = (12, 12, 12), 5
    X = inputs.as_ndarray_view(inputs.uniform(77, 12 ** 3, -1.0, 1.0, dtype=torch.float64), dims)
    A = [inputs.uniform(780 + m, (I, R), -1.0, 1.0).numpy() for m, I in enumerate(dims)]
    for k in range(3):
        ref = oracle.mttkrp(X, A, k)
        good = _einsum_mttkrp(X, A, k)
        assert oracle.normwise_rel_err(good, ref) <= TOL64
        assert oracle.rowwise_rel_err(good, ref) <= TOL64
        bad = _einsum_mttkrp(X, A, k, mutate)
        assert not oracle.normwise_rel_err(bad, ref) <= TOL64, (mutate, k)
        assert not oracle.rowwise_rel_err(bad, ref) <= TOL64, (mutate, k)


def test_gate_rejects_a_wrong_small_row_only_rowwise(oracle):
    """One output row of small norm computed wrongly: the normwise gate lets it through,
    the row-wise gate does not.  (Why the full-size tests assert both.)"""
    import torch
    dims, R = (40, 9, 8), 4
    X = inputs.as_ndarray_view(inputs.uniform(91, 40 * 72, -1.0, 1.0, dtype=torch.float64), dims).copy()
    X[7] *= 1e-9                                  # subtensor 7 of mode 0 is tiny
    A = [inputs.uniform(910 + m, (I, R), -1.0, 1.0).numpy() for m, I in enumerate(dims)]
    ref = oracle.mttkrp(X, A, 0)
    bad = ref.copy()
    bad[7] *= 1.0 + 1e-6
    assert oracle.normwise_rel_err(bad, ref) <= TOL64
    assert not oracle.rowwise_rel_err(bad, ref) <= TOL64
