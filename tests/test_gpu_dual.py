"""GPU parity: cafeq_dual_proxy_loss_fwd_bwd against the oracle."""
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


def _check_dual(env, A, B, T, bits, group, rep, t=5.0, want_codes=True, scale=1.0, flip_slack=False):
    torch, cafeq = env
    P = O.block_inverse(T).astype(np.float32)
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(_dev(torch, A), _dev(torch, B), _dev(torch, T),
                                                       _dev(torch, P), bits, group, rep, t, True, want_codes)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, bits, group, rep, t)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    assert int(losses[5]) == ref["n_groups"] or abs(losses[5] - ref["n_groups"]) <= 1e-6 * ref["n_groups"]
    if flip_slack:
        # hundreds of thousands of groups: a few have two elements within float32 accuracy of the absmax, and
        # the sub-gradient may take either; the bound below is exactly what such a choice can change
        slack, n_amb = parity.dual_argmax_flip_slack(A, B, T, P, ref, group, rep, t)
        print("groups with an ambiguous arg-max: %d of %d" % (n_amb, ref["n_groups"]))
        assert n_amb <= max(3, 1e-4 * ref["n_groups"])
        parity.check_grad_with_slack(grad.cpu().numpy(), ref["gradT"], slack)
    else:
        parity.check_grad(grad.cpu().numpy(), ref["gradT"])
    if want_codes:
        cu, su, cv, sv = [x.cpu().numpy() for x in outs]
        cu_ref, su_ref, _ = O.rtn_sym(ref["U"], bits, group, O.COL)
        cv_ref, sv_ref, _ = O.rtn_sym(ref["V"], bits, group, O.ROW)
        parity.check_scales(su, su_ref)
        parity.check_scales(sv, sv_ref)
        k = T.shape[1]
        unit_u = parity.forward_unit(k, group if group else A.shape[1], bits)
        unit_v = parity.forward_unit(k, group if group else B.shape[0], bits)
        tol_u = parity.tie_tolerance(A, T, O.COL, 1, ref["U"], su_ref, group, unit_u)
        tol_v = parity.tie_tolerance(B, P, O.ROW, rep, ref["V"], sv_ref, group, unit_v)
        parity.check_codes(cu, cu_ref, ref["U"], su_ref, O.COL, group, tie_tol=tol_u)
        parity.check_codes(cv, cv_ref, ref["V"], sv_ref, O.ROW, group, tie_tol=tol_v)


@pytest.mark.parametrize("k,group,rep", [(32, 32, 1), (64, 128, 1), (64, 64, 2), (128, 128, 1), (128, 64, 2)])
def test_dual_small(env, k, group, rep):
    A, B, T = WL.small_pair(200, 512, k, rep, 300 + k + rep, eps=0.05)
    _check_dual(env, A, B, T, 3, group, rep)


def test_dual_large_magnitudes_do_not_overflow_the_exponentials(env):
    # weights scaled so that t * absmax is in the hundreds: exp() of the raw value overflows
    # float32; the running reference must keep everything finite.
    A, B, T = WL.small_pair(200, 256, 64, 1, 333, eps=0.05)
    _check_dual(env, A * 200.0, B * 200.0, T, 4, 64, 1, want_codes=False)


def test_dual_forward_only(env):
    torch, cafeq = env
    A, B, T = WL.small_pair(136, 256, 64, 2, 344, eps=0.05)
    P = O.block_inverse(T).astype(np.float32)
    losses, grad, _ = cafeq.dual_proxy_loss_fwd_bwd(_dev(torch, A), _dev(torch, B), _dev(torch, T),
                                                    _dev(torch, P), 4, 64, 2, 5.0, want_grad=False)
    torch.cuda.synchronize()
    ref = O.dual_lse(A, B, T, P, 4, 64, 2, 5.0, want_grad=False)
    assert grad is None
    parity.check_scalar(float(losses[4]), ref["lse"], what="lse")
    parity.check_scalar(float(losses[2]), ref["l2A_sq"], what="l2A_sq")


def test_config3_full(env):
    c = WL.config3()
    _check_dual(env, c["A"], c["B"], c["T"], 3, 128, 1, want_codes=True)
