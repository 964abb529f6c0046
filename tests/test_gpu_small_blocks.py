"""GPU parity for transform blocks smaller than 32 (the paper's block-size sweep of the single-matrix
hyper-parameter appendix goes down to 2): the library runs a run of 32 / k blocks as one block-diagonal
block of 32; the oracle handles any k natively, so the checks are the usual ones."""
import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL
from tests import parity
from tests.test_gpu_single import _case, _check_single, _dev
from tests.test_gpu_dual import _check_dual

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2511_19705_amd import cafeq
    return torch, cafeq


@pytest.mark.parametrize("k", [2, 4, 8, 16])
def test_block_inverse_small_blocks(env, k):
    torch, cafeq = env
    nb = 3 * (32 // k) * 5
    T = WL.perturbed_blocks(nb, k, 2100 + k, 0.2)
    Tinv, rr, rc, status = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    ref = np.linalg.inv(T.astype(np.float64))
    np.testing.assert_allclose(Tinv.cpu().numpy(), ref, rtol=0, atol=2e-6 * np.abs(ref).max())
    np.testing.assert_allclose(rr.cpu().numpy(), (ref ** 2).sum(axis=2).reshape(-1), rtol=1e-5)
    np.testing.assert_allclose(rc.cpu().numpy(), (ref ** 2).sum(axis=1).reshape(-1), rtol=1e-5)
    assert int(status.abs().sum()) == 0
    # a singular block marks its run of 32 / k blocks, and only that run
    T2 = T.copy()
    T2[1] = 0.0
    Tinv2, status2 = cafeq.block_inverse(_dev(torch, T2))
    torch.cuda.synchronize()
    m = 32 // k
    st = status2.cpu().numpy()
    assert st[:m].all() and not st[m:].any()
    np.testing.assert_allclose(Tinv2.cpu().numpy()[m:], ref[m:], rtol=0, atol=2e-6 * np.abs(ref).max())


@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 1), (O.ROW, 2), (O.ROW, 3)])
@pytest.mark.parametrize("k", [2, 8, 16])
def test_apply_transform_small_blocks(env, axis, rep, k):
    torch, cafeq = env
    W, T, P = _case(axis, 200, 384, k, rep, 2200 + k)
    for side, X in ((cafeq.SIDE_T, T), (cafeq.SIDE_TINV, P)):
        Z = cafeq.apply_transform(_dev(torch, W), _dev(torch, T), _dev(torch, P), axis, side, rep)
        torch.cuda.synchronize()
        ref = O.blockdiag_apply(W, X, axis, rep)
        bound = O.blockdiag_apply(np.abs(W), np.abs(X), axis, rep) * (32 * 2.0 ** -24)
        assert np.all(np.abs(Z.cpu().numpy() - ref) <= bound + 1e-30)


@pytest.mark.parametrize("k,group", [(2, 32), (4, 128), (8, 32), (16, 64), (16, 0), (8, 256)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 2)])
def test_proxy_loss_small_blocks(env, k, group, axis, rep):
    W, T, P = _case(axis, 200, 1024, k, rep, 2300 + k + group)
    _check_single(env, W, T, P, 4, group, axis, rep)


def test_proxy_loss_small_blocks_bf16_minmax_and_forward_only(env):
    torch, cafeq = env
    W, T, P = _case(O.COL, 136, 512, 8, 1, 2401)
    _check_single(env, W, T, P, 3, 64, O.COL, 1, bf16=True)
    from tests.test_gpu_minmax_fused import _check_single_minmax
    _check_single_minmax(env, W, T, P, 4, 128, O.COL, 1)
    losses, grad, _, _ = cafeq.proxy_loss_fwd_bwd(_dev(torch, W), _dev(torch, T), _dev(torch, P), 4, 64, O.COL, want_grad=False)
    torch.cuda.synchronize()
    assert grad is None
    parity.check_scalar(float(losses[0]), O.proxy_l2(W, T, P, 4, 64, O.COL)["l2_sq"], what="l2_sq")


@pytest.mark.parametrize("k,group", [(4, 32), (16, 128), (8, 0)])
def test_dual_small_blocks(env, k, group):
    A, B, T = WL.small_pair(200, 512, k, 1, 2500 + k, eps=0.05)
    _check_dual(env, A, B, T, 4, group, 1)


def test_dual_small_blocks_with_shared_row_blocks_is_refused(env):
    torch, cafeq = env
    A, B, T = WL.small_pair(64, 256, 8, 2, 2550, eps=0.05)
    P = O.block_inverse(T).astype(np.float32)
    with pytest.raises(cafeq.CafeqError):
        cafeq.dual_proxy_loss_fwd_bwd(_dev(torch, A), _dev(torch, B), _dev(torch, T), _dev(torch, P), 4, 32, 2, 5.0)


def test_optimize_single_small_blocks_with_regulariser(env):
    torch, cafeq = env
    W, T, _ = _case(O.COL, 136, 512, 8, 1, 2600, eps=0.0)
    steps, lr, lam = 5, 0.5, 0.05
    Td = _dev(torch, T.copy())
    _, hist, status = cafeq.optimize_single(_dev(torch, W), Td, 4, 64, O.COL, lr=lr, steps=steps, lambda_orth=lam)
    torch.cuda.synchronize()
    T_ref, h_ref = O.optimize_single(W, T, 4, 64, O.COL, 1, lr, steps, lam)
    h = hist.cpu().numpy().astype(np.float64)
    assert int(status.abs().sum()) == 0
    for s in range(steps):
        parity.check_scalar(h[s, 3], h_ref[s, 3], rel=5e-4, what="surrogate at step %d" % s)
        parity.check_scalar(h[s, 4], h_ref[s, 4], rel=5e-4, what="penalty at step %d" % s)
    np.testing.assert_allclose(Td.cpu().numpy(), T_ref, rtol=0, atol=2e-4 * np.abs(T_ref).max())
