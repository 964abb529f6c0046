"""GPU parity for the block and group sizes the paper's experiments use (Sec. 6: blocks of 256 for the
9B model, sub-channel groups of 256, per-channel groups): gradient through the two-pass scheme for
blocks of 256 and groups of 256, and groups that span several segments (whole channels included)
in the single, pair and Alg. 1 entry points."""
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


# (k, group): blocks of 256 with every group size; groups of 256 with smaller blocks
@pytest.mark.parametrize("k,group", [(256, 32), (256, 64), (256, 128), (256, 256), (128, 256), (64, 256), (32, 256)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 1), (O.ROW, 2)])
def test_gradient_for_blocks_and_groups_of_256(env, k, group, axis, rep):
    W, T, P = _case(axis, 200, 1024, k, rep, 700 + k + group)
    _check_single(env, W, T, P, 4, group, axis, rep)


# groups longer than a segment: whole channel (0), a multiple of 128, and a multiple of the block only
@pytest.mark.parametrize("k,group,naxis", [(128, 0, 1024), (256, 0, 1024), (64, 0, 1024), (32, 0, 512),
                                           (128, 512, 1024), (256, 512, 1024), (64, 192, 768), (32, 384, 768)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 2)])
def test_groups_spanning_several_segments(env, k, group, naxis, axis, rep):
    if naxis % (k * rep):
        pytest.skip("axis not divisible by rep blocks")
    W, T, P = _case(axis, 200, naxis, k, rep, 800 + k + group)
    _check_single(env, W, T, P, 4, group, axis, rep)


def test_per_channel_3bit_bf16_and_forward_only(env):
    torch, cafeq = env
    W, T, P = _case(O.COL, 136, 1024, 128, 1, 871)
    _check_single(env, W, T, P, 3, 0, O.COL, 1, bf16=True)
    losses, grad, _, _ = cafeq.proxy_loss_fwd_bwd(_dev(torch, W), _dev(torch, T), _dev(torch, P), 3, 0, O.COL,
                                                  want_grad=False)
    torch.cuda.synchronize()
    ref = O.proxy_l2(W, T, P, 3, 0, O.COL)
    parity.check_scalar(float(losses[0]), ref["l2_sq"], what="l2_sq")
    parity.check_scalar(float(losses[3]), O.surrogate(W, T, P, 3, 0, O.COL, want_grad=False)[0], what="surrogate")


def test_k128_fine_grids_keep_the_six_product_forward(env):
    # 8-bit grid and small groups next to in-line outliers at k = 128: the forward contraction must be
    # accurate to float32 (the two-part half-precision forward is for grids of up to 4 bits)
    for bits, group in ((8, 32), (6, 128), (8, 128)):
        W, T, P = _case(O.COL, 200, 512, 128, 1, 880 + bits + group)
        W[::7, 5] *= 300.0
        _check_single(env, W, T, P, bits, group, O.COL, 1)
        W, T, P = _case(O.ROW, 136, 512, 128, 2, 890 + bits + group)
        _check_single(env, W, T, P, bits, group, O.ROW, 2)


@pytest.mark.parametrize("k,group,rep", [(256, 64, 2), (256, 256, 1), (128, 256, 1), (64, 256, 2),
                                         (128, 0, 1), (256, 0, 2), (64, 0, 2)])
def test_dual_blocks_of_256_and_long_groups(env, k, group, rep):
    A, B, T = WL.small_pair(200, 1024 if rep == 1 else 512, k, rep, 900 + k + rep, eps=0.05)
    _check_dual(env, A, B, T, 4, group, rep)


def test_config4_dual_gradient_full_size(env):
    # the 9B-shaped attention pair at its own block size (per-head 256 x 256 transform, rep 2, group 64, 4 bit)
    c = WL.config4()
    _check_dual(env, c["A"], c["B"], c["T"], 4, 64, 2, want_codes=True, flip_slack=True)
    # and per-channel groups, the setting of the paper's tables on pairs
    _check_dual(env, c["A"], c["B"], c["T"], 4, 0, 2, want_codes=False, flip_slack=True)


@pytest.mark.parametrize("k,group,rep,nb", [(64, 0, 2, 2), (256, 0, 1, 2), (128, 512, 1, 4)])
def test_adaptive_rounding_with_long_groups(env, k, group, rep, nb):
    from tests.test_gpu_adaptive import _pair
    torch, cafeq = env
    bits = 4
    U, V = _pair(328, 296, k, nb, rep, 950 + k)
    cu, su, Uh = O.rtn_sym(U, bits, group, O.COL)
    _, Vh1, Vt, _ = O.adaptive_round_step(U, V, Uh, bits, group, k, rep, half=1)
    cv_ref, sv_ref, _ = O.rtn_sym(Vt, bits, group, O.ROW)
    Ud, Vd = _dev(torch, U), _dev(torch, V)
    dcu, dsu = _dev(torch, cu), _dev(torch, su.astype(np.float32))
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros(sv_ref.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep, half=1)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsv.cpu().numpy(), sv_ref)
    parity.check_codes(dcv.cpu().numpy(), cv_ref, Vt, sv_ref, O.ROW, group)
    # line 4 from the oracle's line-3 result
    _, _, _, Ut = O.adaptive_round_step(U, V, Uh, bits, group, k, rep, half=2, Vh=Vh1)
    cu_ref, su_ref, _ = O.rtn_sym(Ut, bits, group, O.COL)
    dcv2, dsv2 = _dev(torch, cv_ref), _dev(torch, sv_ref.astype(np.float32))
    dcu2 = torch.zeros(U.shape, dtype=torch.int8, device="cuda:0")
    dsu2 = torch.zeros(su_ref.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu2, dsu2, dcv2, dsv2, bits, group, k, rep, half=2)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsu2.cpu().numpy(), su_ref)
    parity.check_codes(dcu2.cpu().numpy(), cu_ref, Ut, su_ref, O.COL, group)


def test_optimize_pair_with_blocks_of_256(env):
    torch, cafeq = env
    A, B, T = WL.small_pair(200, 512, 256, 2, 977, eps=0.0)
    steps, lr = 4, 2e-3
    Td = _dev(torch, T.copy())
    _, hist, status = cafeq.optimize_pair(_dev(torch, A), _dev(torch, B), Td, 4, 64, rep=2, lse_t=5.0, lr=lr, steps=steps)
    torch.cuda.synchronize()
    T_ref, h_ref = O.optimize_pair(A, B, T, 4, 64, 2, 5.0, lr, steps)
    h = hist.cpu().numpy().astype(np.float64)
    for s in range(steps):
        for i in range(5):
            parity.check_scalar(h[s, i], h_ref[s, i], rel=5e-4, what="history[%d][%d]" % (s, i))
    assert np.abs(Td.cpu().numpy() - T_ref).max() <= 3 * lr
