"""Pins for the oracle's randomized-Hadamard baseline."""
import numpy as np
import scipy.linalg

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL


def test_sylvester_matrix_matches_the_library_and_is_orthogonal():
    for n in (1, 2, 8, 64, 1024):
        H = O.hadamard_matrix(n)
        np.testing.assert_array_equal(H, scipy.linalg.hadamard(n))
    H = O.hadamard_matrix(64)
    np.testing.assert_array_equal(H @ H.T, 64 * np.eye(64))
    # entry (i, j) = (-1)^(popcount(i & j)): the closed form of Sylvester's construction
    for i, j in ((3, 5), (7, 7), (12, 10), (63, 21)):
        assert H[i, j] == (-1) ** bin(i & j).count("1")


def test_apply_is_a_rotation_per_block_with_the_signs_on_the_input_side():
    W = WL.gaussian((5, 64), 3).astype(np.float64)
    s = WL.random_signs(64, 4)
    Z = O.hadamard_apply(W, s, 32)
    np.testing.assert_allclose((Z ** 2).sum(axis=1), (W ** 2).sum(axis=1), rtol=1e-12)
    # explicit loops for one row and one block
    H = O.hadamard_matrix(32)
    for j in (0, 9, 31):
        ref = sum(W[2, 32 + l] * s[32 + l] * H[l, j] for l in range(32)) / np.sqrt(32)
        assert abs(Z[2, 32 + j] - ref) < 1e-14
    # a unit vector picks out a signed, normalised row of H
    e = np.zeros((1, 32)); e[0, 5] = 1.0
    np.testing.assert_allclose(O.hadamard_apply(e, s[:32], 32)[0], s[5] * H[5] / np.sqrt(32))


def test_baseline_error_equals_the_rounding_error_and_spreads_outliers():
    W = WL.student_t3((64, 2048), 9)
    WL.scale_random_entries(W, 0.002, 30.0, 10)
    s = WL.random_signs(2048, 11)
    r = O.hadamard_baseline(W, s, 1024, 4, 128)
    assert abs(r["l2_sq"] - r["err_z_sq"]) <= 1e-10 * r["err_z_sq"]
    plain = O.proxy_l2(W, np.eye(32)[None].repeat(64, 0), np.eye(32)[None].repeat(64, 0), 4, 128, O.COL)
    assert r["l2_sq"] < plain["l2_sq"]            # with entry outliers the rotation helps (the paper's premise)
