"""GPU parity of the half-precision forward contraction (128 x 128 blocks, one block per segment): the weights
are scaled per line and the transform per block by powers of two before they are split into two float16 parts,
so results must not depend on magnitudes -- of the whole matrix, of single lines, of the transform -- and lines
of zeros or with a single entry must come out right.  Checked through cafeq_apply_transform (element-wise bound
on Z) and cafeq_proxy_loss_fwd_bwd (codes at the tie rate, scales, losses, gradient) against the oracle."""
import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL
from tests import parity

pytestmark = pytest.mark.gpu
K = 128


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2511_19705_amd import cafeq
    return torch, cafeq


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _blocks(nb, seed, tscale=1.0, eps=0.1):
    T = (WL.perturbed_blocks(nb, K, seed, eps).astype(np.float64) * tscale).astype(np.float32)
    P = O.block_inverse(T).astype(np.float32)
    return T, P


def _check_z(env, W, T, P, axis):
    torch, cafeq = env
    Z = cafeq.apply_transform(_dev(torch, W), _dev(torch, T), _dev(torch, P), axis, cafeq.SIDE_T, 1)
    torch.cuda.synchronize()
    ref = O.blockdiag_apply(W, T, axis, 1)
    bound = O.blockdiag_apply(np.abs(W), np.abs(T), axis, 1) * (K * 2.0 ** -24)
    assert np.all(np.abs(Z.cpu().numpy().astype(np.float64) - ref) <= bound + 1e-300)


def _check_loss(env, W, T, P, bits, group, axis, bf16=False):
    torch, cafeq = env
    if bf16:
        b16 = WL.to_bf16_bits(W)
        W = WL.bf16_bits_to_f32(b16)
        Wd = _dev(torch, b16.view(np.int16)).view(torch.bfloat16)
    else:
        Wd = _dev(torch, W)
    losses, grad, codes, scales = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), bits, group, axis, 1,
                                                           want_grad=True, want_codes=True)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.proxy_l2(W, T, P, bits, group, axis, 1)
    parity.check_scalar(losses[0], ref["l2_sq"], what="l2_sq")
    parity.check_scalar(losses[1], ref["err_z_sq"], what="err_z_sq")
    parity.check_scalar(losses[2], ref["w_sq"], what="w_sq")
    sur, g_ref = O.surrogate(W, T, P, bits, group, axis, 1)
    parity.check_scalar(losses[3], sur, what="surrogate")
    parity.check_grad(grad.cpu().numpy(), g_ref)
    c_ref, s_ref, _ = O.rtn_sym(ref["Z"], bits, group, axis)
    parity.check_scales(scales.cpu().numpy(), s_ref)
    parity.check_codes(codes.cpu().numpy(), c_ref, ref["Z"], s_ref, axis, group)


@pytest.mark.parametrize("wscale", [1e-12, 1.0, 1e12])
@pytest.mark.parametrize("tscale", [1e-3, 1.0, 1e3])
def test_magnitudes_of_the_matrix_and_of_the_transform(env, wscale, tscale):
    T, P = _blocks(3, 11, tscale)
    W = (WL.student_t3((200, 3 * K), 12).astype(np.float64) * wscale).astype(np.float32)
    _check_z(env, W, T, P, O.COL)
    _check_loss(env, W, T, P, 4, 128, O.COL)


@pytest.mark.parametrize("axis", [O.COL, O.ROW])
@pytest.mark.parametrize("group", [32, 128])
def test_lines_of_very_different_magnitudes(env, axis, group):
    rng = np.random.default_rng(21 + group)
    lines, naxis = 168, 2 * K
    T, P = _blocks(2, 22)
    W = WL.student_t3((lines, naxis), 23).astype(np.float64)
    W *= 10.0 ** rng.uniform(-8, 8, (lines, 1))               # every line its own scale
    W[5] = 0.0                                                 # a line of zeros
    W[17] = 0.0; W[17, 200] = 3.0                              # a single entry
    W[40, :K] = 0.0                                            # a segment of zeros next to an ordinary one
    W[41] *= 1e-30 / np.abs(W[41]).max()                       # a very small line (still normal numbers)
    W = W.astype(np.float32)
    if axis == O.ROW:
        W = np.ascontiguousarray(W.T)
    _check_z(env, W, T, P, axis)
    _check_loss(env, W, T, P, 3, group, axis)


def test_entries_of_very_different_magnitudes_within_a_line(env):
    # elements far below the line's largest lose relative, not absolute, accuracy: the bound on Z is absolute
    rng = np.random.default_rng(31)
    T, P = _blocks(2, 32)
    W = WL.student_t3((136, 2 * K), 33).astype(np.float64) * 10.0 ** rng.uniform(-6, 0, (136, 2 * K))
    W = W.astype(np.float32)
    _check_z(env, W, T, P, O.COL)
    _check_loss(env, W, T, P, 4, 64, O.COL)


def test_bfloat16_storage(env):
    T, P = _blocks(2, 41)
    W = WL.student_t3((136, 2 * K), 42)
    _check_loss(env, W, T, P, 4, 128, O.COL, bf16=True)
    _check_loss(env, np.ascontiguousarray(W.T), T, P, 3, 64, O.ROW, bf16=True)


def test_identity_blocks_give_plain_rtn_up_to_ties(env):
    # two float16 parts carry 22 of the 24 bits: Z = W . I is W to 2^-21, so the codes agree with the plain
    # quantizer except, at most, at rounding ties
    torch, cafeq = env
    W = WL.student_t3((200, 4 * K), 51)
    I = np.stack([np.eye(K, dtype=np.float32)] * 4)
    losses, _, codes, scales = cafeq.proxy_loss_fwd_bwd(_dev(torch, W), _dev(torch, I), _dev(torch, I), 4, 128, O.COL,
                                                        want_grad=False, want_codes=True)
    torch.cuda.synchronize()
    c_ref, s_ref, _ = O.rtn_sym(W, 4, 128, O.COL)
    parity.check_scales(scales.cpu().numpy(), s_ref)
    parity.check_codes(codes.cpu().numpy(), c_ref, W.astype(np.float64), s_ref, O.COL, 128)
