"""Pins for the oracle's inference-side function (Sec. 4.1: Y^ = X M^-1 Q(MW))."""
import numpy as np

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL


def _case(out, d, k, bits, group, seed):
    W = WL.student_t3((out, d), seed).astype(np.float64)
    T = WL.perturbed_blocks(d // k, k, seed + 1, eps=0.2).astype(np.float64)
    P = O.block_inverse(T)
    Z = O.blockdiag_apply(W, T, O.COL)
    codes, scales, Zhat = O.rtn_sym(Z, bits, group, O.COL)
    return W, T, P, codes, scales, Zhat


def test_dequantize_reproduces_the_quantizer_output():
    for group in (16, 64, 0):
        W, T, P, codes, scales, Zhat = _case(12, 64, 32, 4, group, 5)
        np.testing.assert_array_equal(O.dequantize(codes, scales, group), Zhat)
    # the other axis
    Z = WL.gaussian((64, 10), 3).astype(np.float64)
    codes, scales, Zhat = O.rtn_sym(Z, 3, 32, O.ROW)
    np.testing.assert_array_equal(O.dequantize(codes, scales, 32, O.ROW), Zhat)


def test_output_equals_the_product_with_the_effective_weight():
    # X M^-1 Q(MW) = X (M^-1 Q(MW)): the effective weight comes from the pinned transform routine
    W, T, P, codes, scales, Zhat = _case(24, 128, 32, 3, 32, 11)
    X = WL.gaussian((5, 128), 12, std=1.0).astype(np.float64)
    West = O.blockdiag_apply(Zhat, P, O.COL)                  # [out][in]
    np.testing.assert_allclose(O.infer_single(X, P, codes, scales, 32), X @ West.T, rtol=1e-12, atol=1e-14)


def test_explicit_loops_on_a_tiny_case():
    W, T, P, codes, scales, Zhat = _case(3, 8, 4, 4, 4, 21)
    X = WL.gaussian((2, 8), 22, std=1.0).astype(np.float64)
    Y = O.infer_single(X, P, codes, scales, 4)
    for t in range(2):
        for o in range(3):
            acc = 0.0
            for i in range(8):                                 # index of the transformed activation
                b = i // 4
                xm = sum(P[b][i % 4][j] * X[t][b * 4 + j] for j in range(4))
                acc += xm * float(np.float32(codes[o][i]) * np.float32(scales[o][i // 4]))
            assert abs(Y[t][o] - acc) < 1e-13


def test_a_weight_on_the_grid_is_reproduced_exactly():
    # Sec. 4.1: with a lossless quantizer M^-1 (MW) = W, the layer output is preserved.  Signed
    # permutations scaled by powers of two are inverted exactly; integer codes with power-of-two scales.
    rng = np.random.default_rng(7)
    nb, k, out, bits, group = 4, 8, 6, 4, 8
    T = np.zeros((nb, k, k))
    for b in range(nb):
        perm = rng.permutation(k)
        T[b][np.arange(k), perm] = rng.choice([-1.0, 1.0], k) * 2.0 ** rng.integers(-1, 2)
    P = O.block_inverse(T)
    q = rng.integers(-7, 8, (out, nb * k))
    q[:, ::group] = 7                                          # the group's absmax sits on the last level
    s = 2.0 ** rng.integers(-4, 0, (out, nb * k // group))
    Zgrid = q * np.repeat(s, group, axis=1)
    W = O.blockdiag_apply(Zgrid, P, O.COL)                     # then W T = Zgrid
    codes, scales, Zhat = O.rtn_sym(O.blockdiag_apply(W, T, O.COL), bits, group, O.COL)
    np.testing.assert_array_equal(Zhat, Zgrid)
    X = rng.integers(-3, 4, (3, nb * k)).astype(np.float64)
    np.testing.assert_array_equal(O.infer_single(X, P, codes, scales, group), X @ W.T)


def test_no_transform_and_identity_transform_coincide():
    W, T, P, codes, scales, Zhat = _case(10, 64, 32, 4, 16, 31)
    X = WL.gaussian((3, 64), 32, std=1.0).astype(np.float64)
    I = np.eye(32)[None].repeat(2, 0)
    np.testing.assert_array_equal(O.infer_single(X, I, codes, scales, 16), O.infer_single(X, None, codes, scales, 16))
    np.testing.assert_allclose(O.infer_single(X, None, codes, scales, 16), X @ Zhat.T, rtol=1e-13)


def test_output_error_is_the_proxy_and_obeys_its_bound():
    # Y^ - Y = X (M^-1 Q(MW) - W): for X = I the squared error is the l2 proxy itself, and for any X
    # the Cauchy-Schwarz bound of Sec. 4.1 holds.
    W, T, P, codes, scales, Zhat = _case(16, 64, 32, 3, 32, 41)
    r = O.proxy_l2(W, T, P, 3, 32, O.COL)
    Yh = O.infer_single(np.eye(64), P, codes, scales, 32)
    assert abs(((Yh - W.T) ** 2).sum() - r["l2_sq"]) <= 1e-10 * r["l2_sq"]
    X = WL.gaussian((7, 64), 42, std=1.0).astype(np.float64)
    err = ((O.infer_single(X, P, codes, scales, 32) - X @ W.T) ** 2).sum()
    assert err <= (X ** 2).sum() * r["l2_sq"]
