"""GPU parity of the loss pass over prepared weights (cafeq_prepare_weights + cafeq_mat::prepared): the same
checks against the oracle as the unprepared path, through the C ABI."""
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


def _check_single_prepared(env, W, T, P, bits, group, axis, rep, bf16=False, want_codes=True, want_grad=True):
    torch, cafeq = env
    if bf16:
        b16 = WL.to_bf16_bits(W)
        W = WL.bf16_bits_to_f32(b16)
        Wd = _dev(torch, b16.view(np.int16)).view(torch.bfloat16)
    else:
        Wd = _dev(torch, W)
    prep = cafeq.prepare_weights(Wd, axis)
    losses, grad, codes, scales = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), bits, group, axis, rep,
                                                           want_grad=want_grad, want_codes=want_codes, prepared=prep)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.proxy_l2(W, T, P, bits, group, axis, rep)
    parity.check_scalar(losses[0], ref["l2_sq"], what="l2_sq")
    parity.check_scalar(losses[1], ref["err_z_sq"], what="err_z_sq")
    parity.check_scalar(losses[2], ref["w_sq"], what="w_sq")
    sur, g_ref = O.surrogate(W, T, P, bits, group, axis, rep, want_grad=want_grad)
    parity.check_scalar(losses[3], sur, what="surrogate")
    if want_grad:
        parity.check_grad(grad.cpu().numpy(), g_ref)
    if want_codes:
        c_ref, s_ref, _ = O.rtn_sym(ref["Z"], bits, group, axis)
        parity.check_scales(scales.cpu().numpy(), s_ref)
        gk = group if group else (W.shape[1] if axis == O.COL else W.shape[0])
        tol = parity.tie_tolerance(W, T, axis, rep, ref["Z"], s_ref, group, parity.forward_unit(T.shape[1], gk, bits))
        parity.check_codes(codes.cpu().numpy(), c_ref, ref["Z"], s_ref, axis, group, tie_tol=tol)


@pytest.mark.parametrize("group", [32, 64, 128])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 1), (O.ROW, 2)])
def test_prepared_single(env, group, axis, rep):
    # 600 lines: two macro-tiles of 256 plus a ragged one (88 lines = two strips + 24 lines); 4 segments
    W, T, P = _case(axis, 600, 512, 128, rep, 1100 + group)
    _check_single_prepared(env, W, T, P, 4, group, axis, rep)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_prepared_bits_bf16_and_forward_only(env, bits):
    W, T, P = _case(O.COL, 200, 256, 128, 1, 1130 + bits)
    _check_single_prepared(env, W, T, P, bits, 128, O.COL, 1, bf16=True)
    W, T, P = _case(O.ROW, 136, 384, 128, 1, 1140 + bits)
    _check_single_prepared(env, W, T, P, bits, 64, O.ROW, 1, want_grad=False, want_codes=False)
    _check_single_prepared(env, W, T, P, bits, 64, O.ROW, 1, want_grad=False, want_codes=True)


def test_prepared_scaled_magnitudes_zero_lines_and_single_entries(env):
    for scale in (1e-12, 1e12):
        W, T, P = _case(O.COL, 300, 256, 128, 1, 1150)
        W = (W.astype(np.float64) * scale).astype(np.float32)
        W[3, :] = 0.0                       # a line of zeros
        W[7, :128] = 0.0
        W[7, 5] = 3.0 * scale               # a segment with a single entry
        _check_single_prepared(env, W, T, P, 4, 64, O.COL, 1)


def test_prepared_falls_back_where_no_kernel_exists(env):
    # blocks of 64 and grids of more than 4 bits have no prepared-weights kernel: the call must give the
    # unprepared path's results (the prepared copy is ignored), not an error
    torch, cafeq = env
    W, T, P = _case(O.COL, 200, 512, 64, 1, 1160)
    Wd = _dev(torch, W)
    prep = cafeq.prepare_weights(Wd, O.COL)
    a = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), 4, 128, O.COL, prepared=prep)
    b = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), 4, 128, O.COL)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    W, T, P = _case(O.COL, 200, 256, 128, 1, 1161)
    _check_single_prepared(env, W, T, P, 8, 128, O.COL, 1)


@pytest.mark.parametrize("group,rep", [(128, 1), (64, 2), (32, 1)])
def test_prepared_dual_small(env, group, rep):
    torch, cafeq = env
    A, B, T = WL.small_pair(600, 512 if rep == 1 else 256, 128, rep, 1170 + group, eps=0.05)
    P = O.block_inverse(T).astype(np.float32)
    Ad, Bd = _dev(torch, A), _dev(torch, B)
    prep = (cafeq.prepare_weights(Ad, O.COL), cafeq.prepare_weights(Bd, O.ROW))
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(Ad, Bd, _dev(torch, T), _dev(torch, P), 3, group, rep, 5.0,
                                                       True, True, prepared=prep)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, 3, group, rep, 5.0)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    assert abs(losses[5] - ref["n_groups"]) <= 1e-6 * ref["n_groups"]
    # a group whose two largest magnitudes agree to float32 accuracy may take either as its arg-max (one of
    # these cases has such a group, gap 1e-7): the bound is exactly what that choice can change
    slack, n_amb = parity.dual_argmax_flip_slack(A, B, T, P, ref, group, rep, 5.0)
    assert n_amb <= 3
    parity.check_grad_with_slack(grad.cpu().numpy(), ref["gradT"], slack)
    cu, su, cv, sv = [x.cpu().numpy() for x in outs]
    cu_ref, su_ref, _ = O.rtn_sym(ref["U"], 3, group, O.COL)
    cv_ref, sv_ref, _ = O.rtn_sym(ref["V"], 3, group, O.ROW)
    parity.check_scales(su, su_ref)
    parity.check_scales(sv, sv_ref)
    parity.check_codes(cu, cu_ref, ref["U"], su_ref, O.COL, group)
    parity.check_codes(cv, cv_ref, ref["V"], sv_ref, O.ROW, group)


def test_prepared_dual_large_magnitudes(env):
    torch, cafeq = env
    A, B, T = WL.small_pair(300, 256, 128, 1, 1180, eps=0.05)
    A, B = A * 200.0, B * 200.0
    P = O.block_inverse(T).astype(np.float32)
    Ad, Bd = _dev(torch, A), _dev(torch, B)
    prep = (cafeq.prepare_weights(Ad, O.COL), cafeq.prepare_weights(Bd, O.ROW))
    losses, grad, _ = cafeq.dual_proxy_loss_fwd_bwd(Ad, Bd, _dev(torch, T), _dev(torch, P), 4, 64, 1, 5.0, True,
                                                    prepared=prep)
    torch.cuda.synchronize()
    ref = O.dual_lse(A, B, T, P, 4, 64, 1, 5.0)
    parity.check_scalar(float(losses[4]), ref["lse"], what="lse")
    parity.check_grad(grad.cpu().numpy(), ref["gradT"])


def test_prepared_config3_full(env):
    """The headline workload through the prepared path, every output against the oracle."""
    torch, cafeq = env
    c = WL.config3()
    A, B, T = c["A"], c["B"], c["T"]
    P = O.block_inverse(T).astype(np.float32)
    Ad, Bd = _dev(torch, A), _dev(torch, B)
    prep = (cafeq.prepare_weights(Ad, O.COL), cafeq.prepare_weights(Bd, O.ROW))
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(Ad, Bd, _dev(torch, T), _dev(torch, P), 3, 128, 1, 5.0,
                                                       True, True, prepared=prep)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, 3, 128, 1, 5.0)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    parity.check_grad(grad.cpu().numpy(), ref["gradT"])
    cu, su, cv, sv = [x.cpu().numpy() for x in outs]
    cu_ref, su_ref, _ = O.rtn_sym(ref["U"], 3, 128, O.COL)
    cv_ref, sv_ref, _ = O.rtn_sym(ref["V"], 3, 128, O.ROW)
    parity.check_scales(su, su_ref)
    parity.check_scales(sv, sv_ref)
    parity.check_codes(cu, cu_ref, ref["U"], su_ref, O.COL, 128)
    parity.check_codes(cv, cv_ref, ref["V"], sv_ref, O.ROW, 128)


def test_prepared_optimize_pair_history(env):
    torch, cafeq = env
    A, B, T = WL.small_pair(300, 256, 128, 1, 1190, eps=0.0)
    steps, lr = 4, 2e-3
    Ad, Bd = _dev(torch, A), _dev(torch, B)
    prep = (cafeq.prepare_weights(Ad, O.COL), cafeq.prepare_weights(Bd, O.ROW))
    Td = _dev(torch, T.copy())
    _, hist, _ = cafeq.optimize_pair(Ad, Bd, Td, 4, 64, rep=1, lse_t=5.0, lr=lr, steps=steps, prepared=prep)
    torch.cuda.synchronize()
    T_ref, h_ref = O.optimize_pair(A, B, T, 4, 64, 1, 5.0, lr, steps)
    h = hist.cpu().numpy().astype(np.float64)
    for s in range(steps):
        for i in range(5):
            parity.check_scalar(h[s, i], h_ref[s, i], rel=5e-4, what="history[%d][%d]" % (s, i))
    assert np.abs(Td.cpu().numpy() - T_ref).max() <= 3 * lr


@pytest.mark.parametrize("bits,group,naxis", [(4, 256, 1024), (4, 0, 1024), (4, 512, 1024), (8, 64, 512)])
@pytest.mark.parametrize("axis,rep", [(O.COL, 1), (O.ROW, 2)])
def test_prepared_gradient_pass_with_the_generic_loss_pass(env, bits, group, naxis, axis, rep):
    # groups of 256, groups that span blocks and fine grids take the loss pass over float32 weights; their
    # gradient pass still reads the prepared copy (blocks of 128)
    W, T, P = _case(axis, 200, naxis, 128, rep, 1700 + bits + group)
    _check_single_prepared(env, W, T, P, bits, group, axis, rep)


def test_prepared_gradient_pass_ragged_lines_and_many_tiles(env):
    # 1000 lines: seven full tiles of 128 and one of 104; more tiles than one workgroup range holds
    W, T, P = _case(O.COL, 1000, 512, 128, 1, 1751)
    _check_single_prepared(env, W, T, P, 3, 128, O.COL, 1, want_codes=False)
    W, T, P = _case(O.ROW, 1000, 512, 128, 2, 1752)
    _check_single_prepared(env, W, T, P, 3, 32, O.ROW, 2, want_codes=False)


@pytest.mark.parametrize("lines", [100, 200, 300, 520])
def test_prepared_pair_with_one_workgroup_per_block(env, lines):
    # 2 x 100 blocks of 128: the call takes the gradient pass that gives every (member, block) a workgroup of its
    # own (its halves take even and odd tiles of 128 lines: 1, 2, 3 and 5 tiles here, the last one ragged), after
    # a single loss launch for both members
    torch, cafeq = env
    A, B, T = WL.small_pair(lines, 12800, 128, 1, 1800 + lines, eps=0.05)
    P = O.block_inverse(T).astype(np.float32)
    Ad, Bd = _dev(torch, A), _dev(torch, B)
    prep = (cafeq.prepare_weights(Ad, O.COL), cafeq.prepare_weights(Bd, O.ROW))
    losses, grad, _ = cafeq.dual_proxy_loss_fwd_bwd(Ad, Bd, _dev(torch, T), _dev(torch, P), 3, 128, 1, 5.0, True, False,
                                                    prepared=prep)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, 3, 128, 1, 5.0)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    slack, n_amb = parity.dual_argmax_flip_slack(A, B, T, P, ref, 128, 1, 5.0)
    assert n_amb <= 3
    parity.check_grad_with_slack(grad.cpu().numpy(), ref["gradT"], slack)


def test_prepared_single_with_one_workgroup_per_block(env):
    # 160 blocks: the single-matrix call takes the same gradient pass (surrogate coefficients)
    for axis, group in ((O.COL, 64), (O.ROW, 128)):
        W, T, P = _case(axis, 200, 20480, 128, 1, 1900 + group)
        _check_single_prepared(env, W, T, P, 4, group, axis, 1, want_codes=False)


def test_prepared_weights_with_padded_rows(env):
    # a view with a leading dimension larger than its width: the preparation reads through it, the passes over the
    # prepared copies never see it
    torch, cafeq = env
    W, T, P = _case(O.COL, 200, 512, 128, 1, 1950)
    big = torch.zeros((200, 640), dtype=torch.float32, device="cuda:0")
    big[:, :512] = _dev(torch, W)
    Wd = big[:, :512]
    assert Wd.stride(0) == 640
    prep = cafeq.prepare_weights(Wd, O.COL)
    losses, grad, _, _ = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), 4, 128, O.COL, prepared=prep)
    torch.cuda.synchronize()
    ref = O.proxy_l2(W, T, P, 4, 128, O.COL)
    parity.check_scalar(float(losses[0]), ref["l2_sq"], what="l2_sq")
    parity.check_scalar(float(losses[2]), ref["w_sq"], what="w_sq")
    parity.check_grad(grad.cpu().numpy(), O.surrogate(W, T, P, 4, 128, O.COL)[1])


def test_launch_timing_samples_every_nth_launch(env):
    # the measurement aid: with every = 3, launches 0, 3, 6, ... of the loss pass are bracketed by the caller's events
    torch, cafeq = env
    W, T, P = _case(O.COL, 200, 512, 128, 1, 1960)
    Wd, Td, Pd = _dev(torch, W), _dev(torch, T), _dev(torch, P)
    timer = cafeq.LaunchTimer(8, every=3)
    with timer:
        for _ in range(7):
            cafeq.proxy_loss_fwd_bwd(Wd, Td, Pd, 4, 128, O.COL, want_grad=False)
        torch.cuda.synchronize()
    assert timer.table.seen == 7 and timer.table.count == 3
    d = timer.durations_ms()
    assert len(d) == 3 and all(x > 0 for x in d)
    # without a table nothing is recorded
    cafeq.proxy_loss_fwd_bwd(Wd, Td, Pd, 4, 128, O.COL, want_grad=False)
    torch.cuda.synchronize()
    assert timer.table.seen == 7
    # kind = 1 brackets the gradient pass instead: one per call with a gradient, none without
    gt = cafeq.LaunchTimer(4, every=1, kind=1)
    with gt:
        cafeq.proxy_loss_fwd_bwd(Wd, Td, Pd, 4, 128, O.COL, want_grad=False)
        cafeq.proxy_loss_fwd_bwd(Wd, Td, Pd, 4, 128, O.COL, want_grad=True)
        cafeq.proxy_loss_fwd_bwd(Wd, Td, Pd, 4, 128, O.COL, want_grad=True)
        torch.cuda.synchronize()
    assert gt.table.seen == 2 and gt.table.count == 2 and all(x > 0 for x in gt.durations_ms())
