"""Pins for the oracle's learning procedure (regulariser, update rules, loops): closed forms,
finite differences and descent properties -- nothing here calls the HIP library."""
import numpy as np

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL


def test_orth_penalty_vanishes_on_rotations_and_matches_the_definition():
    T = WL.haar_blocks(3, 8, 5).astype(np.float64)
    val, g = O.orth_penalty(T, 0.7)
    assert val < 1e-6
    # a scaled rotation c*Q: T T^T - I = (c^2 - 1) I per block -> ||.||_F = |c^2-1| sqrt(d)
    c = 1.3
    val, _ = O.orth_penalty(c * T, 0.7)
    assert abs(val - 0.7 * abs(c * c - 1.0)) < 1e-6
    # explicit loops on a generic block set
    rng = np.random.default_rng(1)
    X = rng.standard_normal((2, 4, 4))
    tot = 0.0
    for b in range(2):
        for i in range(4):
            for j in range(4):
                r = sum(X[b, i, l] * X[b, j, l] for l in range(4)) - (1.0 if i == j else 0.0)
                tot += r * r
    val, _ = O.orth_penalty(X, 2.0)
    assert abs(val - 2.0 * np.sqrt(tot) / np.sqrt(8)) < 1e-12


def test_orth_penalty_gradient_by_finite_differences():
    rng = np.random.default_rng(2)
    T = WL.haar_blocks(2, 6, 9).astype(np.float64) + 0.2 * rng.standard_normal((2, 6, 6))
    _, g = O.orth_penalty(T, 0.5)
    h = 1e-6
    for idx in [(0, 0, 0), (0, 2, 5), (1, 4, 1), (1, 5, 5)]:
        Tp, Tm = T.copy(), T.copy()
        Tp[idx] += h
        Tm[idx] -= h
        fd = (O.orth_penalty(Tp, 0.5)[0] - O.orth_penalty(Tm, 0.5)[0]) / (2 * h)
        assert abs(fd - g[idx]) < 1e-6 * max(1.0, abs(fd))


def test_adam_first_step_is_a_signed_step_of_size_lr():
    # with zero initial moments the bias-corrected first step is lr * g / (|g| + eps)
    g = np.array([[3.0, -0.02], [1e-3, -7.0]])
    T = np.zeros_like(g)
    T1, m, v = O.adam_step(T, g, np.zeros_like(g), np.zeros_like(g), 1, 0.01, 0.1, 0.999, 1e-8)
    np.testing.assert_allclose(T1, -0.01 * np.sign(g), rtol=1e-4)
    np.testing.assert_allclose(m, 0.9 * g)          # (1 - beta1) g with beta1 = 0.1
    np.testing.assert_allclose(v, 1e-3 * g * g)
    # a constant gradient keeps giving steps of size lr (m_hat = g, v_hat = g^2 at every t)
    T2, m, v = O.adam_step(T1, g, m, v, 2, 0.01, 0.1, 0.999, 1e-8)
    np.testing.assert_allclose(T2 - T1, -0.01 * np.sign(g), rtol=1e-4)


def test_gradient_descent_lowers_the_surrogate_and_the_true_error_follows():
    W, T = WL.small_single(96, 128, 32, 61, eps=0.0)
    # outlier columns make the random rotation improvable
    Tn, hist = O.optimize_single(W, T, 4, 32, O.COL, 1, lr=3.0, steps=12)
    sur = hist[:, 3]
    assert np.all(np.diff(sur) < 0)                      # monotone for this step size
    assert sur[-1] < 0.85 * sur[0]
    assert hist[-1, 0] < hist[0, 0]                      # the l2 proxy went down with it
    # normalisation only rescales the step: lr / w_sq without it is the same trajectory
    Tn2, hist2 = O.optimize_single(W, T, 4, 32, O.COL, 1, lr=3.0 / hist[0, 2], steps=12, normalize=False)
    np.testing.assert_allclose(Tn2, Tn, rtol=0, atol=1e-9)


def test_pair_loop_lowers_the_logsumexp_and_regulariser_keeps_t_near_a_rotation():
    A, B, T = WL.small_pair(64, 64, 32, 1, 71)
    Tn, hist = O.optimize_pair(A, B, T, 4, 32, 1, 5.0, lr=1e-2, steps=15)
    assert hist[-1, 4] < hist[0, 4]
    T0, _ = O.optimize_pair(A, B, T, 4, 32, 1, 5.0, lr=1e-2, steps=15, lam=0.0)
    T1, h1 = O.optimize_pair(A, B, T, 4, 32, 1, 5.0, lr=1e-2, steps=15, lam=1.0)
    dev = lambda X: np.sqrt(((X @ X.transpose(0, 2, 1) - np.eye(32)) ** 2).sum())
    assert dev(T1) < dev(T0)
    assert h1[-1, 5] > 0
