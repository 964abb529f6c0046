"""Pins for the oracle's paired transform (LogSumExp surrogate) and Algorithm 1."""
import os

import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold():
    out = {}
    for line in open(os.path.join(GOLD, "toy_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def test_pair_identity_product_preserved():
    A, B, T = WL.small_pair(10, 32, 8, 2, 31, eps=0.3)
    T = T.astype(np.float64)
    P = O.block_inverse(T)
    U = O.blockdiag_apply(A, T, O.COL)
    V = O.blockdiag_apply(B, P, O.ROW, 2)
    for q in range(8):
        b = q // 2
        np.testing.assert_allclose(U[:, b * 8:(b + 1) * 8] @ V[q * 8:(q + 1) * 8],
                                   A[:, b * 8:(b + 1) * 8].astype(np.float64) @ B[q * 8:(q + 1) * 8].astype(np.float64),
                                   atol=1e-12)


def test_lse_literal_formula_bounds_and_limit():
    A, B, T = WL.small_pair(6, 16, 8, 1, 33, eps=0.2)
    T = T.astype(np.float64)
    P = O.block_inverse(T)
    t = 5.0
    out = O.dual_lse(A, B, T, P, 4, 0, 1, t, want_grad=False)
    U, V = out["U"], out["V"]
    # the paper's expression with explicit loops: channel maxima m_u(i), m_v(j)
    tot = 0.0
    for i in range(U.shape[0]):
        tot += np.exp(t * np.max(np.abs(U[i, :])))
    for j in range(V.shape[1]):
        tot += np.exp(t * np.max(np.abs(V[:, j])))
    assert abs(out["lse"] - np.log(tot) / t) < 1e-12
    assert out["n_groups"] == U.shape[0] + V.shape[1]
    mx = max(np.abs(U).max(), np.abs(V).max())
    assert mx <= out["lse"] <= mx + np.log(out["n_groups"]) / t
    big = O.dual_lse(A, B, T, P, 4, 0, 1, 1e4, want_grad=False)["lse"]
    assert abs(big - mx) < 1e-3


def test_dual_errors_are_dense_definitions():
    A, B, T = WL.small_pair(7, 16, 8, 2, 35, eps=0.2)
    T = T.astype(np.float64)
    P = O.block_inverse(T)
    out = O.dual_lse(A, B, T, P, 3, 8, 2, 5.0, arith="f64", want_grad=False)

    def dense(X, rep):
        nb, k, _ = X.shape
        M = np.zeros((nb * rep * k,) * 2)
        for q in range(nb * rep):
            M[q * k:(q + 1) * k, q * k:(q + 1) * k] = X[q // rep]
        return M
    U = A.astype(np.float64) @ dense(T, 1)
    V = dense(P, 2) @ B.astype(np.float64)
    Uh = O.rtn_sym(U, 3, 8, O.COL, "f64")[2]
    Vh = O.rtn_sym(V, 3, 8, O.ROW, "f64")[2]
    np.testing.assert_allclose(out["errU_sq"], ((Uh - U) ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(out["errV_sq"], ((Vh - V) ** 2).sum(), rtol=1e-12)
    np.testing.assert_allclose(out["l2A_sq"], ((Uh @ dense(P, 1) - A) ** 2).sum(), rtol=1e-10)
    np.testing.assert_allclose(out["l2B_sq"], ((dense(T, 2) @ Vh - B) ** 2).sum(), rtol=1e-10)


@pytest.mark.parametrize("k,g,rep", [(8, 8, 1), (8, 4, 2), (4, 8, 2), (8, 0, 1)])
def test_lse_gradient_matches_central_differences(k, g, rep):
    A, B, T = WL.small_pair(5, 16, k, rep, 37, eps=0.4)
    A = A.astype(np.float64) * 30     # make t*absmax O(1) so the softmax is not flat
    B = B.astype(np.float64) * 30
    T = T.astype(np.float64)

    def f(Tx):
        return O.dual_lse(A, B, Tx, O.block_inverse(Tx), 4, g, rep, 5.0, want_grad=False)["lse"]

    grad = O.dual_lse(A, B, T, O.block_inverse(T), 4, g, rep, 5.0)["gradT"]
    fd = np.zeros_like(T)
    h = 1e-6
    it = np.nditer(T, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        Tp = T.copy(); Tp[i] += h
        Tm = T.copy(); Tm[i] -= h
        fd[i] = (f(Tp) - f(Tm)) / (2 * h)
    np.testing.assert_allclose(grad, fd, rtol=2e-5, atol=2e-7 * np.abs(fd).max())


def test_pinv_moore_penrose_identities():
    rng = np.random.default_rng(8)
    for M in (rng.standard_normal((9, 4)), rng.standard_normal((4, 9)),
              rng.standard_normal((6, 3)) @ rng.standard_normal((3, 5))):     # last: rank 3
        X = O.pinv(M)
        np.testing.assert_allclose(M @ X @ M, M, atol=1e-10)
        np.testing.assert_allclose(X @ M @ X, X, atol=1e-10)
        np.testing.assert_allclose((M @ X).T, M @ X, atol=1e-10)
        np.testing.assert_allclose((X @ M).T, X @ M, atol=1e-10)


def test_toy_example_half_iteration():
    g = _gold()
    W = np.diag([g["w_diag0"], g["w_diag1"]])
    bits = int(g["bits"])
    W1h = O.rtn_asym(W, bits, -1, O.COL)[3]
    Uh, Vh, Vt, _ = O.adaptive_round_step(W, W, W1h, bits, -1, k=2, rep=1, half=1, mode=O.ASYM)
    assert abs(Vt[1, 1] - g["target_w2_diag1"]) < 1e-12
    np.testing.assert_allclose(Vh, np.diag([1.0, 0.0]), atol=1e-15)
    p, _ = O.pqe(W, W, Uh, Vh, k=2)
    assert abs(p - g["pqe_after_half_iteration"]) < 1e-12


def test_exactly_representable_first_matrix_reduces_to_plain_quantization():
    rng = np.random.default_rng(9)
    k, d, d3 = 8, 20, 12
    U = rng.integers(-7, 8, size=(d, k)).astype(np.float64)
    U[:, 0] = 7                                           # every group (row) has absmax 7 -> s = 1
    Uh = O.rtn_sym(U, 4, 0, O.COL, "f64")[2]
    np.testing.assert_array_equal(Uh, U)
    V = rng.standard_normal((k, d3))
    _, Vh, Vt, _ = O.adaptive_round_step(U, V, Uh, 4, 0, k, half=1, arith="f64")
    np.testing.assert_allclose(Vt, V, atol=1e-12)
    np.testing.assert_array_equal(Vh, O.rtn_sym(Vt, 4, 0, O.ROW, "f64")[2])


def test_line3_equals_bruteforce_when_gram_is_diagonal():
    rng = np.random.default_rng(10)
    bits = 3
    # k = 1: always separable
    U = rng.standard_normal((9, 1)); Uh = O.rtn_sym(U, bits, 0, O.COL, "f64")[2]
    V = rng.standard_normal((1, 6))
    _, Vh, Vt, _ = O.adaptive_round_step(U, V, Uh, bits, 0, 1, half=1, arith="f64")
    for c in range(6):
        best, _ = O.adaptive_bruteforce_column(Uh, U @ V[:, c], Vt[:, c], bits, 0)
        np.testing.assert_allclose(Vh[:, c], best, atol=1e-14)
    # orthogonal (scaled) columns: separable for any k
    k = 6
    Qm = np.linalg.qr(rng.standard_normal((12, k)))[0] * rng.uniform(0.5, 2.0, size=k)[None, :]
    U = Qm + 0.05 * rng.standard_normal(Qm.shape)
    V = rng.standard_normal((k, 5))
    _, Vh, Vt, _ = O.adaptive_round_step(U, V, Qm, bits, 0, k, half=1, arith="f64")
    for c in range(5):
        best, _ = O.adaptive_bruteforce_column(Qm, U @ V[:, c], Vt[:, c], bits, 0)
        np.testing.assert_allclose(Vh[:, c], best, atol=1e-14)


def test_bruteforce_never_worse_than_step_on_generic_input():
    rng = np.random.default_rng(12)
    k, bits = 8, 3
    U = rng.standard_normal((16, k))
    Uh = O.rtn_sym(U, bits, 0, O.COL, "f64")[2]
    V = rng.standard_normal((k, 4))
    _, Vh, Vt, _ = O.adaptive_round_step(U, V, Uh, bits, 0, k, half=1, arith="f64")
    for c in range(4):
        tgt = U @ V[:, c]
        _, bv = O.adaptive_bruteforce_column(Uh, tgt, Vt[:, c], bits, 0)
        assert bv <= ((Uh @ Vh[:, c] - tgt) ** 2).sum() + 1e-12


def test_adaptive_step_lowers_pqe_on_heavy_tailed_pair():
    A, B, T = WL.small_pair(96, 32, 16, 2, 41)
    T = T.astype(np.float64)
    P = O.block_inverse(T)
    U = O.blockdiag_apply(A, T, O.COL)
    V = O.blockdiag_apply(B, P, O.ROW, 2)
    bits, g = 4, 16
    Uh0 = O.rtn_sym(U, bits, g, O.COL)[2]
    Vh0 = O.rtn_sym(V, bits, g, O.ROW)[2]
    p0, _ = O.pqe(U, V, Uh0, Vh0, 16, 2)
    Uh, Vh = Uh0, None
    for _ in range(3):
        Uh, Vh, _, _ = O.adaptive_round_step(U, V, Uh, bits, g, 16, 2)
    p1, _ = O.pqe(U, V, Uh, Vh, 16, 2)
    assert p1 < 0.95 * p0
