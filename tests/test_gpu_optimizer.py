"""GPU parity: regulariser, update rules and the learning loops against the oracle.

The loops are iterations whose state feeds back: a rounding-level difference in T can flip the
code of an element that sits at a rounding tie, or the arg-max of a group with two nearly equal
maxima, at some later step.  The cases below are small enough that this stays rare and short
enough (about ten steps) that its effect stays far below the tolerances written in each test.
"""
import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2511_19705_amd import cafeq
    return torch, cafeq


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


@pytest.mark.parametrize("k,eps", [(32, 0.2), (64, 0.05), (128, 0.02), (256, 0.1), (64, 0.0)])
def test_orth_penalty(env, k, eps):
    torch, cafeq = env
    T = WL.perturbed_blocks(3, k, 900 + k, eps) if eps else WL.haar_blocks(3, k, 905)
    val_ref, g_ref = O.orth_penalty(T, 0.3)
    base = np.zeros(T.shape, dtype=np.float32)
    base[:, 0, :] = 1.0            # the call increments: these entries keep their offset
    grad = _dev(torch, base.copy())
    val, _ = cafeq.orth_penalty(_dev(torch, T), 0.3, grad)
    torch.cuda.synchronize()
    # the residual is accumulated in float64, so even for a rotation stored in float32 (eps = 0:
    # the residual is pure storage rounding) value and direction follow the oracle
    parity.check_scalar(float(val), val_ref, rel=1e-5, what="penalty")
    got = grad.cpu().numpy().astype(np.float64) - base
    off = base == 0
    assert np.abs(got - g_ref)[off].max() <= 2e-5 * np.abs(g_ref).max()
    assert np.abs(got - g_ref)[~off].max() <= 2e-5 * np.abs(g_ref).max() + 2.0 ** -23   # rounding next to 1.0
    # value only
    val2, _ = cafeq.orth_penalty(_dev(torch, T), 0.3, None)
    assert float(val2) == float(val)


def test_sgd_and_adam_updates(env):
    torch, cafeq = env
    rng = np.random.default_rng(7)
    T = rng.standard_normal((2, 32, 32)).astype(np.float32)
    g = (rng.standard_normal((2, 32, 32)) * 10.0 ** rng.integers(-4, 2, (2, 32, 32))).astype(np.float32)
    Td = _dev(torch, T.copy())
    cafeq.sgd_update(Td, _dev(torch, g), 0.25)
    np.testing.assert_allclose(Td.cpu().numpy(), O.sgd_step(T.astype(np.float64), g, 0.25), rtol=1e-6, atol=1e-7)
    den = _dev(torch, np.array([4.0], dtype=np.float32))
    Td = _dev(torch, T.copy())
    cafeq.sgd_update(Td, _dev(torch, g), 0.25, den)
    np.testing.assert_allclose(Td.cpu().numpy(), O.sgd_step(T.astype(np.float64), g / 4.0, 0.25), rtol=1e-6, atol=1e-7)
    # three Adam steps with changing gradients
    Td = _dev(torch, T.copy())
    m = torch.zeros_like(Td)
    v = torch.zeros_like(Td)
    Tr, mr, vr = T.astype(np.float64), np.zeros(T.shape), np.zeros(T.shape)
    for t in range(1, 4):
        gt = (g * (1.0 + 0.5 * t) * (-1.0) ** t).astype(np.float32)
        cafeq.adam_update(Td, _dev(torch, gt), m, v, t, 1e-2, 0.1, 0.999, 1e-8)
        Tr, mr, vr = O.adam_step(Tr, gt.astype(np.float64), mr, vr, t, 1e-2, 0.1, 0.999, 1e-8)
    torch.cuda.synchronize()
    np.testing.assert_allclose(Td.cpu().numpy(), Tr, rtol=2e-6, atol=2e-7)
    np.testing.assert_allclose(m.cpu().numpy(), mr, rtol=1e-5, atol=1e-12)
    np.testing.assert_allclose(v.cpu().numpy(), vr, rtol=1e-5, atol=1e-20)


@pytest.mark.parametrize("axis,k,group,lam,normalize", [(O.COL, 32, 32, 0.0, True), (O.COL, 64, 128, 0.5, True),
                                                         (O.ROW, 128, 64, 0.0, True), (O.COL, 128, 128, 0.2, False)])
def test_single_matrix_gradient_descent_follows_the_oracle(env, axis, k, group, lam, normalize):
    torch, cafeq = env
    steps = 8
    lines, naxis = 200, 256
    T0 = WL.perturbed_blocks(naxis // k, k, 950 + k, 0.03)
    W = WL.student_t3((lines, naxis) if axis == O.COL else (naxis, lines), 951 + k)
    WL.scale_random_entries(W, 0.002, 20.0, 952)
    lr = 2.0 if normalize else 2.0 / float((W.astype(np.float64) ** 2).sum())
    T_ref, h_ref = O.optimize_single(W, T0, 4, group, axis, 1, lr, steps, lam, normalize)
    Td = _dev(torch, T0.copy())
    Tinv, hist, status = cafeq.optimize_single(_dev(torch, W), Td, 4, group, axis, 1, lr, steps, lam, normalize)
    torch.cuda.synchronize()
    hist = hist.cpu().numpy().astype(np.float64)
    assert int(status.abs().sum()) == 0
    for s in range(steps):
        for c, name in enumerate(("l2_sq", "err_z_sq", "w_sq", "surrogate", "penalty")):
            parity.check_scalar(hist[s, c], h_ref[s, c], rel=5e-4, what="step %d %s" % (s, name))
    assert h_ref[-1, 3] < h_ref[0, 3] and hist[-1, 3] < hist[0, 3]   # the descent is real
    Tg = Td.cpu().numpy().astype(np.float64)
    assert np.abs(Tg - T_ref).max() <= 2e-4 * np.abs(T_ref).max()
    np.testing.assert_allclose(Tinv.cpu().numpy(), np.linalg.inv(Tg), rtol=0, atol=1e-5 * np.abs(np.linalg.inv(Tg)).max())


@pytest.mark.parametrize("k,group,rep,lam", [(32, 32, 1, 0.0), (64, 64, 2, 0.1), (128, 128, 1, 1.0)])
def test_pair_adam_follows_the_oracle(env, k, group, rep, lam):
    torch, cafeq = env
    steps = 8
    A, B, T0 = WL.small_pair(136, 256, k, rep, 970 + k, eps=0.03)
    T_ref, h_ref = O.optimize_pair(A, B, T0, 4, group, rep, 5.0, 3e-3, steps, lam)
    Td = _dev(torch, T0.copy())
    Tinv, hist, status = cafeq.optimize_pair(_dev(torch, A), _dev(torch, B), Td, 4, group, rep, 5.0, 3e-3, steps, lam)
    torch.cuda.synchronize()
    hist = hist.cpu().numpy().astype(np.float64)
    assert int(status.abs().sum()) == 0
    for s in range(steps):
        for c, name in ((0, "errU_sq"), (1, "errV_sq"), (2, "l2A_sq"), (3, "l2B_sq"), (4, "lse")):
            parity.check_scalar(hist[s, c], h_ref[s, c], rel=5e-4, what="step %d %s" % (s, name))
        parity.check_scalar(hist[s, 6], h_ref[s, 5], rel=5e-4, what="step %d penalty" % s)
    Tg = Td.cpu().numpy().astype(np.float64)
    # Adam's step is lr * sign-like: an entry whose tiny gradient differs in the last float32 bits
    # may move by up to lr per step in another direction; bound by a few steps' worth
    assert np.abs(Tg - T_ref).max() <= 3 * 3e-3
    assert np.sqrt(((Tg - T_ref) ** 2).mean()) <= 1e-4


@pytest.mark.parametrize("k,lr", [(64, 6e-3), (128, 6e-3), (64, 2e-2), (128, 2e-2)])
def test_pair_adam_with_large_steps_follows_the_oracle(env, k, lr):
    """Inside the loop the inverse is warm-started from the previous iteration's; steps this large make the
    warm start take all its rounds (k = 64 at 6e-3) or hand the block to the elimination (the others)."""
    torch, cafeq = env
    steps = 5
    A, B, T0 = WL.small_pair(136, 256, k, 1, 990 + k, eps=0.03)
    T_ref, h_ref = O.optimize_pair(A, B, T0, 4, k, 1, 5.0, lr, steps, 0.1)
    Td = _dev(torch, T0.copy())
    Tinv, hist, status = cafeq.optimize_pair(_dev(torch, A), _dev(torch, B), Td, 4, k, 1, 5.0, lr, steps, 0.1)
    torch.cuda.synchronize()
    hist = hist.cpu().numpy().astype(np.float64)
    assert int(status.abs().sum()) == 0
    for s in range(steps):
        for c, name in ((0, "errU_sq"), (1, "errV_sq"), (2, "l2A_sq"), (3, "l2B_sq"), (4, "lse")):
            parity.check_scalar(hist[s, c], h_ref[s, c], rel=5e-4, what="step %d %s" % (s, name))
    Tg = Td.cpu().numpy().astype(np.float64)
    assert np.sqrt(((Tg - T_ref) ** 2).mean()) <= 0.05 * lr
    np.testing.assert_allclose(Tinv.cpu().numpy(), np.linalg.inv(Tg), rtol=0, atol=1e-5 * np.abs(np.linalg.inv(Tg)).max())


@pytest.mark.parametrize("lr,rep", [(3e-3, 1), (6e-3, 2)])
def test_pair_adam_with_blocks_of_256_follows_the_oracle(env, lr, rep):
    """Blocks of 256 (the paper's setting for the 9B model): inside the loop the inverse comes from Newton-Schulz
    rounds started at the previous iteration's inverse, with the elimination behind them."""
    torch, cafeq = env
    k, steps = 256, 5
    A, B, T0 = WL.small_pair(136, 512, k, rep, 1256 + rep, eps=0.03)
    T_ref, h_ref = O.optimize_pair(A, B, T0, 4, 64, rep, 5.0, lr, steps, 0.1)
    Td = _dev(torch, T0.copy())
    Tinv, hist, status = cafeq.optimize_pair(_dev(torch, A), _dev(torch, B), Td, 4, 64, rep, 5.0, lr, steps, 0.1)
    torch.cuda.synchronize()
    hist = hist.cpu().numpy().astype(np.float64)
    assert int(status.abs().sum()) == 0
    for s in range(steps):
        for c, name in ((0, "errU_sq"), (1, "errV_sq"), (2, "l2A_sq"), (3, "l2B_sq"), (4, "lse")):
            parity.check_scalar(hist[s, c], h_ref[s, c], rel=5e-4, what="step %d %s" % (s, name))
    Tg = Td.cpu().numpy().astype(np.float64)
    assert np.sqrt(((Tg - T_ref) ** 2).mean()) <= 0.05 * lr
    np.testing.assert_allclose(Tinv.cpu().numpy(), np.linalg.inv(Tg), rtol=0, atol=1e-5 * np.abs(np.linalg.inv(Tg)).max())


def test_learning_on_the_bench_workload_lowers_the_loss(env):
    """Ten Adam steps on the full 9B-shaped pair: the LogSumExp falls, nothing is singular.
    (Size-independent property; the small cases above carry the element-wise parity.)"""
    torch, cafeq = env
    c = WL.config3()
    Td = _dev(torch, c["T"].copy())
    Tinv, hist, status = cafeq.optimize_pair(_dev(torch, c["A"]), _dev(torch, c["B"]), Td, 3, 128, 1, 5.0, 1e-3, 10)
    torch.cuda.synchronize()
    hist = hist.cpu().numpy()
    assert int(status.abs().sum()) == 0
    assert np.all(np.isfinite(hist))
    assert hist[-1, 4] < hist[0, 4]
