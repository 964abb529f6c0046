"""GPU parity for the min/max grid of the paper's Eq. (1) inside the loss / gradient path
(cfg->mode = CAFEQ_Q_ASYM_MINMAX): losses, the surrogate with the constant the paper prints
(1 / (2^b - 1)^2, Sec. 4.1) and its gradient, codes, scales and minima, for single matrices and pairs,
groups inside a segment and groups that span segments (whole channels included)."""
import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL
from tests import parity
from tests.test_gpu_single import _case, _dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2511_19705_amd import cafeq
    return torch, cafeq


def _check_single_minmax(env, W, T, P, bits, group, axis, rep, bf16=False, want_grad=True):
    torch, cafeq = env
    if bf16:
        b16 = WL.to_bf16_bits(W)
        W = WL.bf16_bits_to_f32(b16)
        Wd = _dev(torch, b16.view(np.int16)).view(torch.bfloat16)
    else:
        Wd = _dev(torch, W)
    losses, grad, codes, scales = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), bits, group, axis, rep,
                                                           want_grad=want_grad, want_codes=True, mode=cafeq.Q_MINMAX)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.proxy_l2(W, T, P, bits, group, axis, rep, mode=O.ASYM)
    parity.check_scalar(losses[0], ref["l2_sq"], what="l2_sq")
    parity.check_scalar(losses[1], ref["err_z_sq"], what="err_z_sq")
    parity.check_scalar(losses[2], ref["w_sq"], what="w_sq")
    sur, g_ref = O.surrogate(W, T, P, bits, group, axis, rep, mode=O.ASYM, want_grad=want_grad)
    parity.check_scalar(losses[3], sur, what="surrogate")
    if want_grad:
        parity.check_grad(grad.cpu().numpy(), g_ref)
    c_ref, s_ref, lo_ref, _ = O.rtn_asym(ref["Z"], bits, group, axis, "f32")
    sc = scales.cpu().numpy()
    assert codes.dtype == torch.uint8 and sc.shape == (2,) + s_ref.shape
    parity.check_scales(sc[0], s_ref)
    parity.check_mins(sc[1], lo_ref, s_ref, 2 ** bits - 1)
    # (here the scale moves with the errors at the group's minimum and maximum: twice the arg-max term bounds both)
    tol = 2.0 * parity.tie_tolerance(W, T, axis, rep, ref["Z"], s_ref, group, parity.UNIT_FULL)
    parity.check_codes_minmax(codes.cpu().numpy(), c_ref, ref["Z"], s_ref, lo_ref, axis, group, tie_tol=tol)


@pytest.mark.parametrize("k,group", [(32, 32), (32, 128), (64, 128), (64, 32), (128, 128), (128, 64), (256, 256),
                                     (256, 64), (128, 256)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 2)])
def test_minmax_single(env, k, group, axis, rep):
    W, T, P = _case(axis, 200, 1024, k, rep, 1100 + k + group)
    _check_single_minmax(env, W, T, P, 4, group, axis, rep)


@pytest.mark.parametrize("k,group,naxis", [(128, 0, 1024), (256, 0, 1024), (64, 0, 1024), (32, 384, 768), (128, 512, 1024)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 2)])
def test_minmax_groups_spanning_several_segments(env, k, group, naxis, axis, rep):
    if naxis % (k * rep):
        pytest.skip("axis not divisible by rep blocks")
    W, T, P = _case(axis, 200, naxis, k, rep, 1200 + k + group)
    _check_single_minmax(env, W, T, P, 4, group, axis, rep)


@pytest.mark.parametrize("bits", [2, 3, 8])
def test_minmax_bits_bf16_and_forward_only(env, bits):
    W, T, P = _case(O.COL, 136, 512, 64, 1, 1300 + bits)
    _check_single_minmax(env, W, T, P, bits, 128, O.COL, 1)
    _check_single_minmax(env, W, T, P, bits, 128, O.COL, 1, bf16=True, want_grad=False)
    W, T, P = _case(O.ROW, 136, 512, 128, 1, 1310 + bits)
    _check_single_minmax(env, W, T, P, bits, 0, O.ROW, 1, bf16=True)


def test_minmax_constant_groups_and_positive_lines(env):
    # lines of zeros (range 0: code 0, value = minimum), and lines that are positive throughout -- where the
    # grid of Eq. (1) differs most from the symmetric one
    W, T, P = _case(O.COL, 136, 512, 64, 1, 1331)
    W[5] = 0.0
    W[40:48] = 0.0
    W[60:70] = np.abs(W[60:70]) + 0.05
    I = np.stack([np.eye(64, dtype=np.float32)] * 8)
    _check_single_minmax(env, W, I, I, 4, 64, O.COL, 1)
    _check_single_minmax(env, W, T, P, 4, 128, O.COL, 1)


def _check_dual_minmax(env, A, B, T, bits, group, rep, t=5.0):
    torch, cafeq = env
    P = O.block_inverse(T).astype(np.float32)
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(_dev(torch, A), _dev(torch, B), _dev(torch, T), _dev(torch, P),
                                                       bits, group, rep, t, True, True, mode=cafeq.Q_MINMAX)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, bits, group, rep, t, mode=O.ASYM)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    parity.check_grad(grad.cpu().numpy(), ref["gradT"])
    cu, su, cv, sv = [x.cpu().numpy() for x in outs]
    for codes, sc, Z, axis in ((cu, su, ref["U"], O.COL), (cv, sv, ref["V"], O.ROW)):
        c_ref, s_ref, lo_ref, _ = O.rtn_asym(Z, bits, group, axis, "f32")
        parity.check_scales(sc[0], s_ref)
        parity.check_mins(sc[1], lo_ref, s_ref, 2 ** bits - 1)
        parity.check_codes_minmax(codes, c_ref, Z, s_ref, lo_ref, axis, group)


@pytest.mark.parametrize("k,group,rep", [(64, 64, 2), (128, 128, 1), (256, 64, 2), (128, 0, 1), (32, 32, 1)])
def test_minmax_dual(env, k, group, rep):
    A, B, T = WL.small_pair(200, 1024 if rep == 1 else 512, k, rep, 1400 + k + rep, eps=0.05)
    _check_dual_minmax(env, A, B, T, 4, group, rep)


def test_minmax_optimize_single_first_step(env):
    # the learning loop passes the grid through: its first recorded losses are those of the single call
    torch, cafeq = env
    W, T, P = _case(O.COL, 136, 512, 64, 1, 1500)
    Td = _dev(torch, T.copy())
    _, hist, _ = cafeq.optimize_single(_dev(torch, W), Td, 4, 128, O.COL, lr=0.5, steps=3, mode=cafeq.Q_MINMAX)
    torch.cuda.synchronize()
    h = hist.cpu().numpy().astype(np.float64)
    ref = O.proxy_l2(W, T, P, 4, 128, O.COL, mode=O.ASYM)
    parity.check_scalar(h[0, 0], ref["l2_sq"], what="l2_sq")
    parity.check_scalar(h[0, 3], O.surrogate(W, T, P, 4, 128, O.COL, mode=O.ASYM, want_grad=False)[0], what="surrogate")
    assert h[2, 3] < h[0, 3]
