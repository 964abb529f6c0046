"""Pins for the oracle's block-diagonal transform, l2 proxy and surrogate."""
import os

import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def dense_blockdiag(X, rep=1):
    nb, k, _ = X.shape
    n = nb * rep * k
    M = np.zeros((n, n))
    for q in range(nb * rep):
        M[q * k:(q + 1) * k, q * k:(q + 1) * k] = X[q // rep]
    return M


def naive_matmul(A, B):
    n, m = A.shape
    m2, p = B.shape
    out = np.zeros((n, p))
    for i in range(n):
        for j in range(p):
            acc = 0.0
            for l in range(m):
                acc += A[i, l] * B[l, j]
            out[i, j] = acc
    return out


def test_apply_equals_dense_triple_loop():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((3, 4, 4))
    W = rng.standard_normal((5, 12))
    np.testing.assert_allclose(O.blockdiag_apply(W, X, O.COL), naive_matmul(W, dense_blockdiag(X)), atol=1e-13)
    W2 = rng.standard_normal((24, 5))
    np.testing.assert_allclose(O.blockdiag_apply(W2, X, O.ROW, rep=2),
                               naive_matmul(dense_blockdiag(X, 2), W2), atol=1e-13)


@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 1), (O.ROW, 2)])
def test_no_quantization_identity_and_orthogonal_norm(axis, rep):
    # M^-1 (M W) - W = 0; a rotation preserves the Frobenius norm
    k, nb = 16, 3
    T = WL.perturbed_blocks(nb, k, 3, eps=0.3).astype(np.float64)
    P = O.block_inverse(T)
    shape = (20, nb * k) if axis == O.COL else (nb * rep * k, 20)
    W = np.random.default_rng(1).standard_normal(shape)
    Z = O.blockdiag_apply(W, T, axis, rep)
    np.testing.assert_allclose(O.blockdiag_apply(Z, P, axis, rep), W, atol=1e-11)
    Q = WL.haar_blocks(nb, k, 4).astype(np.float64)
    ZQ = O.blockdiag_apply(W, Q, axis, rep)
    assert abs(np.linalg.norm(ZQ) - np.linalg.norm(W)) < 1e-5 * np.linalg.norm(W)


def test_orthogonal_transform_l2_equals_transformed_error():
    W, T = WL.small_single(48, 128, 32, 7)
    T = T.astype(np.float64)
    # re-orthogonalise in float64 so that P = T^T to 1e-15
    T = np.stack([np.linalg.qr(t)[0] for t in T])
    out = O.proxy_l2(W, T, T.transpose(0, 2, 1), 4, 32, O.COL)
    assert abs(out["l2_sq"] - out["err_z_sq"]) < 1e-10 * out["err_z_sq"]


def test_identity_transform_is_plain_rtn():
    W, _ = WL.small_single(40, 128, 32, 8)
    I = np.stack([np.eye(32)] * 4)
    out = O.proxy_l2(W, I, I, 4, 64, O.COL)
    codes, scales, what = O.rtn_sym(W, 4, 64, O.COL)
    np.testing.assert_array_equal(out["Zhat"], what)
    assert abs(out["l2_sq"] - ((what - W.astype(np.float64)) ** 2).sum()) < 1e-18
    # more bits -> the proxy goes to zero
    l8 = O.proxy_l2(W, I, I, 8, 64, O.COL)["l2_sq"]
    assert l8 < out["l2_sq"] / 100


def test_l2_proxy_is_dense_definition():
    # || Q(W T) P - W ||_F^2 assembled from dense matrices
    W, T = WL.small_single(12, 32, 8, 9, eps=0.2)
    T = T.astype(np.float64)
    P = O.block_inverse(T)
    out = O.proxy_l2(W, T, P, 3, 16, O.COL, arith="f64")
    Z = W.astype(np.float64) @ dense_blockdiag(T)
    Zh = O.rtn_sym(Z, 3, 16, O.COL, "f64")[2]
    D = Zh @ dense_blockdiag(P) - W
    assert abs(out["l2_sq"] - (D ** 2).sum()) < 1e-12 * (D ** 2).sum()


def test_surrogate_reproduces_printed_bound():
    # paper orientation: W_io is d1 x d2 (y = x W), M = blockdiag(M_b) acts on d1.
    rng = np.random.default_rng(2)
    d1, d2, k, bits = 12, 7, 4, 3
    Mb = rng.standard_normal((3, k, k)) + 2 * np.eye(k)
    M = dense_blockdiag(Mb)
    W_io = rng.standard_normal((d1, d2))
    printed = O.surrogate_printed(W_io, M, bits)
    # this repo's layout: W = W_io^T ([out][in]), transform on the columns with T = M^T
    T = Mb.transpose(0, 2, 1)
    P = O.block_inverse(T)
    got, _ = O.surrogate(W_io.T.copy(), T, P, bits, 0, O.COL, mode=O.ASYM,
                         group_axis=O.ROW, want_grad=False)
    assert abs(got - printed) < 1e-12 * printed


def test_surrogate_orthogonal_closed_form():
    W, T = WL.small_single(24, 64, 16, 12)
    T = np.stack([np.linalg.qr(t.astype(np.float64))[0] for t in T])
    P = T.transpose(0, 2, 1)
    g, bits = 32, 4
    got, _ = O.surrogate(W, T, P, bits, g, O.COL, want_grad=False)
    Z = O.blockdiag_apply(W, T, O.COL)
    a = np.abs(Z.reshape(24, 2, g)).max(axis=2)
    assert abs(got - (g * a ** 2).sum() / (4 * 7 * 7)) < 1e-12 * got


@pytest.mark.parametrize("axis", [O.COL, O.ROW])
def test_surrogate_bounds_expected_error_under_stochastic_rounding(axis):
    # E||P-applied error||^2 for independent zero-mean rounding errors equals
    # sum_e rho_j(e) Var_e  (this fixes which norms of P enter rho), and the
    # surrogate upper-bounds it.  Checked analytically and by simulation.
    rng = np.random.default_rng(4)
    k, nb, g, bits = 8, 2, 8, 3
    T = WL.perturbed_blocks(nb, k, 5, eps=0.4).astype(np.float64)
    P = O.block_inverse(T)
    W = rng.standard_normal((6, nb * k)) if axis == O.COL else rng.standard_normal((nb * k, 6))
    Z = O.blockdiag_apply(W, T, axis)
    qmax = 2 ** (bits - 1) - 1
    Zg = O._to_groups(Z, axis, g)
    s = np.abs(Zg).max(axis=1, keepdims=True) / qmax
    x = Zg / s
    lo = np.floor(x)
    f = x - lo
    var_g = s ** 2 * f * (1 - f)
    var = O._from_groups(var_g, Z.shape, axis, g)
    rho = O.rho_from_inverse(P, axis)
    expected = (var * (rho[None, :] if axis == O.COL else rho[:, None])).sum()
    sur, _ = O.surrogate(W, T, P, bits, g, axis, want_grad=False)
    assert expected <= sur
    acc, n = 0.0, 3000
    for _ in range(n):
        up = rng.random(x.shape) < f
        Zh = O._from_groups((lo + up) * s, Z.shape, axis, g)
        D = O.blockdiag_apply(Zh - Z, P, axis)
        acc += (D ** 2).sum()
    assert abs(acc / n - expected) < 0.05 * expected


def _fd_grad(fun, T, h=1e-6):
    g = np.zeros_like(T)
    it = np.nditer(T, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        Tp = T.copy(); Tp[i] += h
        Tm = T.copy(); Tm[i] -= h
        g[i] = (fun(Tp) - fun(Tm)) / (2 * h)
    return g


@pytest.mark.parametrize("axis,rep,k,g", [(O.COL, 1, 8, 8), (O.COL, 1, 8, 4), (O.COL, 1, 4, 8),
                                           (O.ROW, 1, 8, 8), (O.ROW, 2, 4, 8), (O.ROW, 2, 8, 4)])
@pytest.mark.parametrize("mode", [O.SYM, O.ASYM])
def test_surrogate_gradient_matches_central_differences(axis, rep, k, g, mode):
    rng = np.random.default_rng(6)
    nb = 2
    T = WL.perturbed_blocks(nb, k, 13, eps=0.5).astype(np.float64)
    W = rng.standard_normal((9, nb * k)) if axis == O.COL else rng.standard_normal((nb * rep * k, 9))

    def f(Tx):
        return O.surrogate(W, Tx, O.block_inverse(Tx), 4, g, axis, rep, mode, want_grad=False)[0]

    _, grad = O.surrogate(W, T, O.block_inverse(T), 4, g, axis, rep, mode)
    fd = _fd_grad(f, T)
    np.testing.assert_allclose(grad, fd, rtol=2e-5, atol=2e-7 * np.abs(fd).max())


def test_table1_extra_flops_closed_form():
    # cost model of the block-diagonal inverse: k / 9216 (percent), Hadamard: log2(n)/9216
    for line in open(os.path.join(GOLD, "table1_extra_flops.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, printed = line.split()
        val = 100.0 * (np.log2(1024) if name.startswith("hadamard") else float(name)) / 9216
        assert abs(val - float(printed)) <= 0.005 + 1e-12
