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


@pytest.mark.parametrize("mode", [O.SYM, O.ASYM])
def test_dual_errors_are_dense_definitions(mode):
    A, B, T = WL.small_pair(7, 16, 8, 2, 35, eps=0.2)
    T = T.astype(np.float64)
    P = O.block_inverse(T)
    out = O.dual_lse(A, B, T, P, 3, 8, 2, 5.0, arith="f64", want_grad=False, mode=mode)
    sym_lse = O.dual_lse(A, B, T, P, 3, 8, 2, 5.0, arith="f64", want_grad=False)["lse"]
    assert out["lse"] == sym_lse          # a function of the group maxima alone

    def dense(X, rep):
        nb, k, _ = X.shape
        M = np.zeros((nb * rep * k,) * 2)
        for q in range(nb * rep):
            M[q * k:(q + 1) * k, q * k:(q + 1) * k] = X[q // rep]
        return M
    U = A.astype(np.float64) @ dense(T, 1)
    V = dense(P, 2) @ B.astype(np.float64)
    if mode == O.SYM:
        Uh = O.rtn_sym(U, 3, 8, O.COL, "f64")[2]
        Vh = O.rtn_sym(V, 3, 8, O.ROW, "f64")[2]
    else:
        # Eq. (1) with explicit loops over the groups
        def eq1(X):
            out_ = np.empty_like(X)
            for i in range(X.shape[0]):
                for g0 in range(0, X.shape[1], 8):
                    x = X[i, g0:g0 + 8]
                    s_ = (x.max() - x.min()) / 7.0
                    out_[i, g0:g0 + 8] = s_ * np.rint((x - x.min()) / s_) + x.min()
            return out_
        Uh = eq1(U)
        Vh = eq1(V.T).T
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


# ---------------------------------------------------------------------------------------------
# Algorithm 1, line 4 (the update of the first matrix) and the paired error over several heads
# ---------------------------------------------------------------------------------------------
def _stack_heads(X, k, b, rep):
    """Row-blocks b*rep .. (b+1)*rep-1 of X (k rows each) side by side, with explicit loops."""
    d3 = X.shape[1]
    out = np.zeros((k, rep * d3))
    for r in range(rep):
        for i in range(k):
            for c in range(d3):
                out[i, r * d3 + c] = X[(b * rep + r) * k + i, c]
    return out


def test_line4_is_line3_of_the_transposed_pair():
    # W1 W2 Vh^+ = (Vh^T^+ W2^T W1^T)^T: line 4 on (U, V, Vh) is the transpose of line 3 on
    # (V^T, U^T, Vh^T); line 3 is pinned by the paper's toy example and by brute force above
    rng = np.random.default_rng(21)
    k, nb, d1, d3 = 6, 3, 11, 9
    U = rng.standard_normal((d1, nb * k))
    V = rng.standard_normal((nb * k, d3))
    Vh = O.rtn_sym(V, 3, 0, O.ROW, "f64")[2]
    got = O.adaptive_targets_U(U, V, Vh, k, 1)
    want = O.adaptive_targets_V(V.T, Vh.T, U.T, k, 1).T
    np.testing.assert_allclose(got, want, atol=1e-11)
    # and the full step (with its quantizer on the other axis) obeys the same symmetry
    Uh0 = O.rtn_sym(U, 3, 0, O.COL, "f64")[2]
    Uh4, _, _, Ut = O.adaptive_round_step(U, V, Uh0, 3, 0, k, 1, half=2, Vh=Vh, arith="f64")
    _, Vh3, Vt, _ = O.adaptive_round_step(V.T, U.T, Vh.T, 3, 0, k, 1, half=1, arith="f64")
    np.testing.assert_allclose(Ut, Vt.T, atol=1e-11)
    np.testing.assert_allclose(Uh4, Vh3.T, atol=1e-11)


def test_line4_normal_equations_with_shared_heads():
    # U'_b is the least-squares solution of X Vh_[b] = U_b V_[b] over the rep row-blocks of head b
    # side by side: residual times Vh_[b]^T vanishes.  Everything formed with explicit loops.
    rng = np.random.default_rng(22)
    k, nb, rep, d1, d3 = 4, 2, 2, 5, 7
    U = rng.standard_normal((d1, nb * k))
    V = rng.standard_normal((nb * rep * k, d3))
    Vh = O.rtn_sym(V, 3, 0, O.ROW, "f64")[2]
    Ut = O.adaptive_targets_U(U, V, Vh, k, rep)
    for b in range(nb):
        Vs, Vhs = _stack_heads(V, k, b, rep), _stack_heads(Vh, k, b, rep)
        for i in range(d1):
            for j in range(k):
                acc = 0.0
                for c in range(rep * d3):
                    got = sum(Ut[i, b * k + l] * Vhs[l, c] for l in range(k))
                    ref = sum(U[i, b * k + l] * Vs[l, c] for l in range(k))
                    acc += (got - ref) * Vhs[j, c]
                assert abs(acc) < 1e-10, (b, i, j, acc)
        # the same solution from a different library routine (least squares on the transposed system)
        X = np.linalg.lstsq(Vhs.T, (U[:, b * k:(b + 1) * k] @ Vs).T, rcond=None)[0].T
        np.testing.assert_allclose(Ut[:, b * k:(b + 1) * k], X, atol=1e-10)
        # a wrong stacking (heads added instead of placed side by side) is a different matrix
        wrong = U[:, b * k:(b + 1) * k] @ (sum(V[q * k:(q + 1) * k] for q in range(b * rep, (b + 1) * rep))
                                           @ O.pinv(sum(Vh[q * k:(q + 1) * k] for q in range(b * rep, (b + 1) * rep))))
        assert np.abs(wrong - Ut[:, b * k:(b + 1) * k]).max() > 1e-3


def test_line4_no_perturbation_lowers_the_paired_error():
    rng = np.random.default_rng(23)
    k, nb, rep, d1, d3 = 4, 2, 2, 6, 5
    U = rng.standard_normal((d1, nb * k))
    V = rng.standard_normal((nb * rep * k, d3))
    Vh = O.rtn_sym(V, 3, 0, O.ROW, "f64")[2]
    Ut = O.adaptive_targets_U(U, V, Vh, k, rep)
    base = O.pqe(U, V, Ut, Vh, k, rep)[0]
    for _ in range(50):
        assert O.pqe(U, V, Ut + 1e-3 * rng.standard_normal(Ut.shape), Vh, k, rep)[0] >= base - 1e-12


def test_toy_example_second_half_iteration_by_hand():
    # Not printed in the paper; worked by hand from Algorithm 1, line 4 on the Sec. 5 toy example after
    # its first half-iteration:  W1 W2 = diag(1, 0.36),  W2^ = diag(1, 0),  pinv(W2^) = diag(1, 0),
    # target = diag(1, 0.36) diag(1, 0) = diag(1, 0),  Q(target) = diag(1, 0) on the 1-bit grid {0, 1};
    # the paired error stays ||diag(1,0) diag(1,0) - diag(1,0.36)||_F = 0.36.
    g = _gold()
    W = np.diag([g["w_diag0"], g["w_diag1"]])
    bits = int(g["bits"])
    W1h = O.rtn_asym(W, bits, -1, O.COL)[3]
    Uh, Vh, _, Ut = O.adaptive_round_step(W, W, W1h, bits, -1, k=2, rep=1, half=0, mode=O.ASYM)
    np.testing.assert_allclose(Ut, np.diag([1.0, 0.0]), atol=1e-15)
    np.testing.assert_allclose(Uh, np.diag([1.0, 0.0]), atol=1e-15)
    np.testing.assert_allclose(Vh, np.diag([1.0, 0.0]), atol=1e-15)
    assert abs(O.pqe(W, W, Uh, Vh, k=2)[0] - 0.36) < 1e-12
    # a non-commuting case by hand: W1 = [[1, 1], [0, 1]], W2 = I, W2^ = diag(2, 1):
    # W1 W2 pinv(W2^) = [[1/2, 1], [0, 1]]  (the pseudoinverse on the right scales COLUMNS)
    W1 = np.array([[1.0, 1.0], [0.0, 1.0]])
    got = O.adaptive_targets_U(W1, np.eye(2), np.diag([2.0, 1.0]), 2, 1)
    np.testing.assert_allclose(got, np.array([[0.5, 1.0], [0.0, 1.0]]), atol=1e-15)


def test_line4_exactly_representable_second_matrix_reduces_to_plain_quantization():
    rng = np.random.default_rng(24)
    k, rep, d3 = 5, 2, 6
    V = rng.integers(-3, 4, size=(rep * k, d3)).astype(np.float64)
    V[0, :] = 3                                       # every column group of each row-block has absmax 3
    V[k, :] = -3
    Vh = O.rtn_sym(V, 3, k, O.ROW, "f64")[2]
    np.testing.assert_array_equal(Vh, V)
    U = rng.standard_normal((9, k))
    Uh, _, _, Ut = O.adaptive_round_step(U, V, None, 3, k, k, rep, half=2, Vh=Vh, arith="f64")
    np.testing.assert_allclose(Ut, U, atol=1e-11)      # V_[b] has full row rank: U V pinv(V) = U
    np.testing.assert_array_equal(Uh, O.rtn_sym(Ut, 3, k, O.COL, "f64")[2])


def test_line4_equals_bruteforce_when_rows_of_the_second_matrix_are_orthogonal():
    rng = np.random.default_rng(25)
    bits, k, rep, d3 = 3, 5, 2, 7
    # orthogonal (scaled) rows of the stacked quantized matrix: the problem separates per entry of a row of U'
    Qm = np.linalg.qr(rng.standard_normal((rep * d3, k)))[0].T * rng.uniform(0.5, 2.0, size=k)[:, None]   # k x rep*d3
    Vh = np.concatenate([Qm[:, r * d3:(r + 1) * d3] for r in range(rep)], axis=0)                         # rep*k x d3
    V = Vh + 0.05 * rng.standard_normal(Vh.shape)
    U = rng.standard_normal((4, k))
    Uh, _, _, Ut = O.adaptive_round_step(U, V, None, bits, 0, k, rep, half=2, Vh=Vh, arith="f64")
    Vs = _stack_heads(V, k, 0, rep)
    for i in range(U.shape[0]):
        best, _ = O.adaptive_bruteforce_column(Qm.T, (U[i] @ Vs), Ut[i], bits, 0)
        np.testing.assert_allclose(Uh[i], best, atol=1e-13)


def test_pqe_over_shared_heads_is_the_dense_loop():
    rng = np.random.default_rng(26)
    k, nb, rep, d1, d3 = 3, 2, 2, 4, 5
    U = rng.standard_normal((d1, nb * k)); Uh = U + 0.1 * rng.standard_normal(U.shape)
    V = rng.standard_normal((nb * rep * k, d3)); Vh = V + 0.1 * rng.standard_normal(V.shape)
    num = den = 0.0
    for q in range(nb * rep):
        b = q // rep
        for i in range(d1):
            for c in range(d3):
                ref = sum(U[i, b * k + l] * V[q * k + l, c] for l in range(k))
                got = sum(Uh[i, b * k + l] * Vh[q * k + l, c] for l in range(k))
                num += (got - ref) ** 2
                den += ref ** 2
    p, rel = O.pqe(U, V, Uh, Vh, k, rep)
    assert abs(p - np.sqrt(num)) < 1e-12 and abs(rel - np.sqrt(num / den)) < 1e-12
    # rep = 1 with one head is the plain Frobenius norm of the product difference
    p1, _ = O.pqe(U[:, :k], V[:k], Uh[:, :k], Vh[:k], k, 1)
    assert abs(p1 - np.linalg.norm(Uh[:, :k] @ Vh[:k] - U[:, :k] @ V[:k])) < 1e-12
