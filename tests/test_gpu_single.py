"""GPU parity: cafeq_apply_transform and cafeq_proxy_loss_fwd_bwd against the oracle."""
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


def _case(axis, lines, naxis, k, rep, seed, eps=0.05):
    nb = naxis // (k * rep)
    T = WL.perturbed_blocks(nb, k, seed + 1, eps) if eps else WL.haar_blocks(nb, k, seed + 1)
    shape = (lines, naxis) if axis == O.COL else (naxis, lines)
    W = WL.student_t3(shape, seed)
    if axis == O.COL:
        WL.scale_random_columns(W, 2, 10.0, seed + 2)
    else:
        WL.scale_random_entries(W, 0.001, 20.0, seed + 2)
    P = O.block_inverse(T).astype(np.float32)
    return W, T, P


@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 1), (O.ROW, 2)])
@pytest.mark.parametrize("k", [32, 64, 128, 256])
def test_apply_transform(env, axis, rep, k):
    torch, cafeq = env
    W, T, P = _case(axis, 200, 512, k, rep, 40 + k)
    for side, X in ((cafeq.SIDE_T, T), (cafeq.SIDE_TINV, P)):
        Z = cafeq.apply_transform(_dev(torch, W), _dev(torch, T), _dev(torch, P), axis, side, rep)
        torch.cuda.synchronize()
        ref = O.blockdiag_apply(W, X, axis, rep)
        bound = O.blockdiag_apply(np.abs(W), np.abs(X), axis, rep) * (k * 2.0 ** -24)
        assert np.all(np.abs(Z.cpu().numpy() - ref) <= bound + 1e-30)


def _check_single(env, W, T, P, bits, group, axis, rep, bf16=False, want_codes=True):
    torch, cafeq = env
    if bf16:
        b16 = WL.to_bf16_bits(W)
        W = WL.bf16_bits_to_f32(b16)
        Wd = _dev(torch, b16.view(np.int16)).view(torch.bfloat16)
    else:
        Wd = _dev(torch, W)
    losses, grad, codes, scales = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), bits, group,
                                                           axis, rep, want_grad=True, want_codes=want_codes)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.proxy_l2(W, T, P, bits, group, axis, rep)
    parity.check_scalar(losses[0], ref["l2_sq"], what="l2_sq")
    parity.check_scalar(losses[1], ref["err_z_sq"], what="err_z_sq")
    parity.check_scalar(losses[2], ref["w_sq"], what="w_sq")
    sur, g_ref = O.surrogate(W, T, P, bits, group, axis, rep)
    parity.check_scalar(losses[3], sur, what="surrogate")
    parity.check_grad(grad.cpu().numpy(), g_ref)
    if want_codes:
        c_ref, s_ref, _ = O.rtn_sym(ref["Z"], bits, group, axis)
        parity.check_scales(scales.cpu().numpy(), s_ref)
        k = T.shape[1]
        gk = group if group else (W.shape[1] if axis == O.COL else W.shape[0])
        tol = parity.tie_tolerance(W, T, axis, rep, ref["Z"], s_ref, group, parity.forward_unit(k, gk, bits))
        parity.check_codes(codes.cpu().numpy(), c_ref, ref["Z"], s_ref, axis, group, tie_tol=tol)


@pytest.mark.parametrize("k,group", [(32, 32), (32, 128), (64, 128), (64, 32), (128, 128), (128, 64)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 1), (O.ROW, 2)])
def test_proxy_loss_small(env, k, group, axis, rep):
    # 200 lines: one full macro-tile of 128 plus a ragged one (72 = two strips + 8 lines)
    W, T, P = _case(axis, 200, 1024, k, rep, 60 + k + group)
    _check_single(env, W, T, P, 4, group, axis, rep)


@pytest.mark.parametrize("bits", [2, 3, 8])
def test_proxy_loss_bits_and_bf16(env, bits):
    W, T, P = _case(O.COL, 136, 512, 64, 1, 80 + bits)
    _check_single(env, W, T, P, bits, 128, O.COL, 1)
    _check_single(env, W, T, P, bits, 128, O.COL, 1, bf16=True)
    W, T, P = _case(O.ROW, 136, 512, 64, 1, 90 + bits)
    _check_single(env, W, T, P, bits, 64, O.ROW, 1, bf16=True)


def test_identity_transform_reduces_to_plain_rtn(env):
    torch, cafeq = env
    W = WL.student_t3((96, 512), 7)
    I = np.stack([np.eye(64, dtype=np.float32)] * 8)
    losses, _, codes, scales = cafeq.proxy_loss_fwd_bwd(_dev(torch, W), _dev(torch, I), _dev(torch, I), 4, 128,
                                                        O.COL, want_grad=False, want_codes=True)
    c2, s2, err = cafeq.rtn_quantize(_dev(torch, W), 4, 128, O.COL, want_err=True)
    torch.cuda.synchronize()
    assert torch.equal(codes, c2) and torch.equal(scales, s2)
    c_ref, s_ref, _ = O.rtn_sym(W, 4, 128, O.COL)
    np.testing.assert_array_equal(codes.cpu().numpy(), c_ref)
    parity.check_scalar(float(losses[0]), float(err), rel=1e-5, what="l2 == rtn error")


def test_config1_full(env):
    c = WL.config1()
    P = O.block_inverse(c["T"]).astype(np.float32)
    _check_single(env, c["W"], c["T"], P, 4, 32, O.COL, 1)


def test_config2_full(env):
    c = WL.config2()
    P = O.block_inverse(c["T"]).astype(np.float32)
    for bits in c["bits"]:
        _check_single(env, c["W"], c["T"], P, bits, 128, O.COL, 1)


def test_unsupported_and_bad_arguments(env):
    torch, cafeq = env
    W = torch.zeros((64, 512), device="cuda:0")
    T = torch.eye(64, device="cuda:0").repeat(8, 1, 1).contiguous()
    with pytest.raises(cafeq.CafeqError):
        cafeq.proxy_loss_fwd_bwd(W, T, T, 4, 48, O.COL)          # group not supported by the fused kernel
    with pytest.raises(cafeq.CafeqError):
        cafeq.apply_transform(W[:, :448], T, T, O.COL)           # cols != nb*k
    with pytest.raises(cafeq.CafeqError):
        cafeq.proxy_loss_fwd_bwd(W, T, T, 1, 128, O.COL)         # bits out of range
