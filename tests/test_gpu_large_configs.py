"""GPU parity at the full sizes of the attention pair (config 4, adaptive rounding, k = 256) and of
the 27B-shaped layer (config 5, bfloat16 storage, k = 128): the launch configurations the library
picks for these shapes, checked against the oracle.

Where the oracle finishes in seconds the whole output is compared (q, k, the V/O pairs).  For the
three 170 M-element matrices (gate, down, up) the oracle is evaluated on what it can compute one
piece at a time -- sampled lines (a line's codes and scale depend on that line only), sampled
transform blocks (a block's gradient depends on its slab only) -- and the scalars are checked
through identities that hold at any size, evaluated in float64 from device outputs whose samples
were just compared with the oracle.
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


def _dev_bf16(torch, bits16):
    return _dev(torch, bits16.view(np.int16)).view(torch.bfloat16)


def _dequant(codes, scales, group, axis):
    return codes.astype(np.float64) * np.repeat(scales.astype(np.float64), group, axis=1 if axis == O.COL else 0)


def _sample(n, count, seed):
    """First two, last two and `count` random indices of range(n), sorted."""
    rng = np.random.default_rng(seed)
    idx = set([0, 1, n - 2, n - 1]) | set(rng.choice(n, size=count, replace=False).tolist())
    return np.array(sorted(idx))


# ------------------------------------------------------------------------------------------
# config 4: V/O pair of a 9B-shaped attention layer, k = 256, rep = 2, group 64, 4 bit
# ------------------------------------------------------------------------------------------
def test_config4_transform_and_adaptive_step_full_size(env):
    torch, cafeq = env
    c = WL.config4()
    A, B, T, k, rep, group, bits = c["A"], c["B"], c["T"], c["k"], c["rep"], c["group"], c["bits"][0]
    P = O.block_inverse(T)
    U64 = O.blockdiag_apply(A, T, O.COL)
    V64 = O.blockdiag_apply(B, P, O.ROW, rep)
    Td, Pd = _dev(torch, T), _dev(torch, P.astype(np.float32))
    # S1 at this shape (k = 256 forward-only kernel), both members
    Ug = cafeq.apply_transform(_dev(torch, A), Td, Pd, O.COL, cafeq.SIDE_T, 1).cpu().numpy()
    Vg = cafeq.apply_transform(_dev(torch, B), Td, Pd, O.ROW, cafeq.SIDE_TINV, rep).cpu().numpy()
    bu = O.blockdiag_apply(np.abs(A), np.abs(T), O.COL) * (k * 2.0 ** -24)
    bv = O.blockdiag_apply(np.abs(B), np.abs(P), O.ROW, rep) * (k * 2.0 ** -24)
    assert np.all(np.abs(Ug - U64) <= bu + 1e-30)
    assert np.all(np.abs(Vg - V64) <= bv + 1e-30)

    # Alg. 1, each line from the oracle's state (inputs are the oracle's U, V rounded to float32)
    U, V = U64.astype(np.float32), V64.astype(np.float32)
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    Uh = _dequant(cu, su, group, O.COL)
    _, _, Vt, Ut = O.adaptive_round_step(U, V, Uh, bits, group, k, rep, half=0)
    cv_ref, sv_ref, _ = O.rtn_sym(Vt, bits, group, O.ROW)
    cu_ref, su_ref, _ = O.rtn_sym(Ut, bits, group, O.COL)
    Ud, Vd = _dev(torch, U), _dev(torch, V)
    dcu, dsu = _dev(torch, cu), _dev(torch, su.astype(np.float32))
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros(sv_ref.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep, half=1)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsv.cpu().numpy(), sv_ref)
    parity.check_codes(dcv.cpu().numpy(), cv_ref, Vt, sv_ref, O.ROW, group)
    dcv2, dsv2 = _dev(torch, cv_ref), _dev(torch, sv_ref.astype(np.float32))
    dcu2 = torch.zeros(U.shape, dtype=torch.int8, device="cuda:0")
    dsu2 = torch.zeros(su_ref.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu2, dsu2, dcv2, dsv2, bits, group, k, rep, half=2)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsu2.cpu().numpy(), su_ref)
    parity.check_codes(dcu2.cpu().numpy(), cu_ref, Ut, su_ref, O.COL, group)


def test_config4_paired_quantization_error_full_size(env):
    """PQE of the independently rounded attention pair: Gram-trace evaluation on the device against
    the oracle's d1 x d3 products."""
    torch, cafeq = env
    c = WL.config4()
    A, B, T, k, rep, group, bits = c["A"], c["B"], c["T"], c["k"], c["rep"], c["group"], c["bits"][0]
    P = O.block_inverse(T)
    U = O.blockdiag_apply(A, T, O.COL).astype(np.float32)
    V = O.blockdiag_apply(B, P, O.ROW, rep).astype(np.float32)
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    cv, sv, _ = O.rtn_sym(V, bits, group, O.ROW)
    p_abs, p_rel = O.pqe(U, V, _dequant(cu, su, group, O.COL), _dequant(cv, sv, group, O.ROW), k, rep)
    out = cafeq.pqe(_dev(torch, U), _dev(torch, V), _dev(torch, cu), _dev(torch, su.astype(np.float32)),
                    _dev(torch, cv), _dev(torch, sv.astype(np.float32)), bits, group, k, rep)
    out = out.cpu().numpy().astype(np.float64)
    parity.check_scalar(out[0], p_abs ** 2, what="pqe_sq")
    parity.check_scalar(np.sqrt(out[0] / out[1]), p_rel, what="relative pqe")


def test_config4_dual_forward_full_size(env):
    """The pair's losses at k = 256 without the gradient (the gradient at full size: test_gpu_long_groups.py)."""
    torch, cafeq = env
    c = WL.config4()
    A, B, T, rep, group, bits = c["A"], c["B"], c["T"], c["rep"], c["group"], c["bits"][0]
    P = O.block_inverse(T).astype(np.float32)
    losses, grad, _ = cafeq.dual_proxy_loss_fwd_bwd(_dev(torch, A), _dev(torch, B), _dev(torch, T), _dev(torch, P),
                                                    bits, group, rep, 5.0, want_grad=False)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, bits, group, rep, 5.0, want_grad=False)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)


# ------------------------------------------------------------------------------------------
# config 5: 27B-shaped layer, bfloat16 storage, k = 128, group 128
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,bits", [("q", 3), ("k", 4)])
def test_config5_single_full_oracle(env, name, bits):
    torch, cafeq = env
    t = WL.config5_tensor(name)
    W = WL.bf16_bits_to_f32(t["bits16"])
    T = WL.config5_transform("single")
    P = O.block_inverse(T).astype(np.float32)
    losses, grad, codes, scales = cafeq.proxy_loss_fwd_bwd(_dev_bf16(torch, t["bits16"]), _dev(torch, T),
                                                           _dev(torch, P), bits, 128, O.COL, 1,
                                                           want_grad=True, want_codes=True)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.proxy_l2(W, T, P, bits, 128, O.COL, 1)
    parity.check_scalar(losses[0], ref["l2_sq"], what="l2_sq")
    parity.check_scalar(losses[1], ref["err_z_sq"], what="err_z_sq")
    parity.check_scalar(losses[2], ref["w_sq"], what="w_sq")
    sur, g_ref = O.surrogate(W, T, P, bits, 128, O.COL, 1)
    parity.check_scalar(losses[3], sur, what="surrogate")
    parity.check_grad(grad.cpu().numpy(), g_ref)
    c_ref, s_ref, _ = O.rtn_sym(ref["Z"], bits, 128, O.COL)
    parity.check_scales(scales.cpu().numpy(), s_ref)
    parity.check_codes(codes.cpu().numpy(), c_ref, ref["Z"], s_ref, O.COL, 128)


def test_config5_gate_sampled(env):
    """gate 36864 x 4608 (170 M elements, bfloat16), 3 bit: sampled rows and blocks + identities."""
    torch, cafeq = env
    bits, group, k = 3, 128, 128
    t = WL.config5_tensor("gate")
    T = WL.config5_transform("single")
    P64 = O.block_inverse(T)
    P = P64.astype(np.float32)
    Wd = _dev_bf16(torch, t["bits16"])
    losses, grad, codes, scales = cafeq.proxy_loss_fwd_bwd(Wd, _dev(torch, T), _dev(torch, P), bits, group,
                                                           O.COL, 1, want_grad=True, want_codes=True)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    nrows = t["bits16"].shape[0]
    # (1) sampled rows: codes and scales of a row depend on that row only
    rows = _sample(nrows, 92, 5101)
    Ws = WL.bf16_bits_to_f32(t["bits16"][rows])
    Zs = O.blockdiag_apply(Ws, T, O.COL)
    c_ref, s_ref, _ = O.rtn_sym(Zs, bits, group, O.COL)
    rows_d = torch.from_numpy(rows).to("cuda:0")
    parity.check_scales(scales[rows_d].cpu().numpy(), s_ref)
    parity.check_codes(codes[rows_d].cpu().numpy(), c_ref, Zs, s_ref, O.COL, group)
    # (2) ||W||^2 exactly; T is orthogonal to float32 rounding, so ||D||^2 = ||E||^2 (rotation
    #     invariance of the Frobenius norm) to the same accuracy
    w_sq = 0.0
    for r0 in range(0, nrows, 4096):
        w_sq += float((WL.bf16_bits_to_f32(t["bits16"][r0:r0 + 4096]).astype(np.float64) ** 2).sum())
    parity.check_scalar(losses[2], w_sq, what="w_sq")
    parity.check_scalar(losses[0], losses[1], rel=2e-5, what="l2_sq vs err_z_sq under an orthogonal transform")
    # (3) the surrogate from its definition, with the group maxima taken from the device scales
    #     (a_G = s_G * qmax up to one float32 rounding) and rho from the oracle's inverse
    qmax = 2 ** (bits - 1) - 1
    a2 = (scales.cpu().numpy().astype(np.float64) * qmax) ** 2            # [rows][groups]
    rho = O.rho_from_inverse(P64, O.COL)                                   # [nb*k]
    rG = rho.reshape(-1, group).sum(axis=1)
    sur = O.beta_const(bits, O.SYM) * float((a2 * rG[None, :]).sum())
    parity.check_scalar(losses[3], sur, rel=1e-5, what="surrogate from device scales")
    # (4) sampled blocks of the gradient: block b depends on column slab b only
    g = grad.cpu().numpy()
    for b in (0, 17, 35):
        Wb = WL.bf16_bits_to_f32(np.ascontiguousarray(t["bits16"][:, b * k:(b + 1) * k]))
        _, g_ref = O.surrogate(Wb, T[b:b + 1], P[b:b + 1], bits, group, O.COL, 1)
        parity.check_grad(g[b:b + 1], g_ref)


@pytest.mark.parametrize("bits,prepared", [(3, False), (4, False), (3, True)])
def test_config5_mlp_pair_sampled(env, bits, prepared):
    """down 4608 x 36864 (T on its columns) with up 36864 x 4608 (T^-1 on its rows), 288 blocks; both bit
    widths of the layer protocol, and the loss pass over prepared weights."""
    torch, cafeq = env
    group, k, t_lse = 128, 128, 5.0
    ta, tb = WL.config5_tensor("down"), WL.config5_tensor("up")
    T = WL.config5_transform("mlp")
    P64 = O.block_inverse(T)
    P = P64.astype(np.float32)
    Ad, Bd = _dev_bf16(torch, ta["bits16"]), _dev_bf16(torch, tb["bits16"])
    prep = (cafeq.prepare_weights(Ad, cafeq.AXIS_COL), cafeq.prepare_weights(Bd, cafeq.AXIS_ROW)) if prepared else (None, None)
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(Ad, Bd, _dev(torch, T), _dev(torch, P), bits, group, 1, t_lse,
                                                       True, True, prepared=prep)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    cu, su, cv, sv = outs
    # (1) sampled rows of A and sampled columns of B
    rows = _sample(ta["bits16"].shape[0], 60, 5201)
    As = WL.bf16_bits_to_f32(ta["bits16"][rows])
    Us = O.blockdiag_apply(As, T, O.COL)
    c_ref, s_ref, _ = O.rtn_sym(Us, bits, group, O.COL)
    rd = torch.from_numpy(rows).to("cuda:0")
    parity.check_scales(su[rd].cpu().numpy(), s_ref)
    parity.check_codes(cu[rd].cpu().numpy(), c_ref, Us, s_ref, O.COL, group)
    cols = _sample(tb["bits16"].shape[1], 60, 5202)
    Bs = WL.bf16_bits_to_f32(np.ascontiguousarray(tb["bits16"][:, cols]))
    Vs = O.blockdiag_apply(Bs, P64, O.ROW, 1)
    c_ref, s_ref, _ = O.rtn_sym(Vs, bits, group, O.ROW)
    cd = torch.from_numpy(cols).to("cuda:0")
    parity.check_scales(sv[:, cd].cpu().numpy(), s_ref)
    parity.check_codes(cv[:, cd].cpu().numpy(), c_ref, Vs, s_ref, O.ROW, group)
    # (2) LogSumExp over every group of both members from the device scales
    qmax = 2 ** (bits - 1) - 1
    a = np.concatenate([su.cpu().numpy().ravel(), sv.cpu().numpy().ravel()]).astype(np.float64) * qmax
    m = a.max()
    lse = m + np.log(np.exp(t_lse * (a - m)).sum()) / t_lse
    parity.check_scalar(losses[4], lse, rel=1e-6, what="lse from device scales")
    assert int(round(losses[5])) == a.size
    # (3) T orthogonal to float32 rounding: the proxy equals the rounding error of each member
    parity.check_scalar(losses[2], losses[0], rel=2e-5, what="l2A_sq vs errU_sq")
    parity.check_scalar(losses[3], losses[1], rel=2e-5, what="l2B_sq vs errV_sq")
    # (4) sampled blocks of the gradient.  Block b sees only column slab b of A and row slab b of
    #     B, except for the softmax normalisation: the oracle on the slab pair normalises by the
    #     slab's own sum of exponentials, so its gradient is the full one times exp(t (lse - lse_b)).
    g = grad.cpu().numpy()
    for b in (0, 143, 287):
        Ab = WL.bf16_bits_to_f32(np.ascontiguousarray(ta["bits16"][:, b * k:(b + 1) * k]))
        Bb = WL.bf16_bits_to_f32(tb["bits16"][b * k:(b + 1) * k])
        ref = O.dual_lse(Ab, Bb, T[b:b + 1], P[b:b + 1], bits, group, 1, t_lse)
        g_ref = ref["gradT"] * np.exp(t_lse * (ref["lse"] - lse))
        parity.check_grad(g[b:b + 1], g_ref)


def test_config5_vo_pair_3bit_full_oracle(env):
    """The same pair at the layer protocol's other bit width: paired losses, gradient and codes."""
    torch, cafeq = env
    bits, group, rep = 3, 128, 2
    ta, tb = WL.config5_tensor("v"), WL.config5_tensor("o")
    A, B = WL.bf16_bits_to_f32(ta["bits16"]), WL.bf16_bits_to_f32(tb["bits16"])
    T = WL.config5_transform("vo")
    P = O.block_inverse(T).astype(np.float32)
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(_dev_bf16(torch, ta["bits16"]), _dev_bf16(torch, tb["bits16"]),
                                                       _dev(torch, T), _dev(torch, P), bits, group, rep, 5.0,
                                                       True, True)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, bits, group, rep, 5.0)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    parity.check_grad(grad.cpu().numpy(), ref["gradT"])
    cu, su, cv, sv = [x.cpu().numpy() for x in outs]
    cu_ref, su_ref, _ = O.rtn_sym(ref["U"], bits, group, O.COL)
    cv_ref, sv_ref, _ = O.rtn_sym(ref["V"], bits, group, O.ROW)
    parity.check_scales(su, su_ref)
    parity.check_scales(sv, sv_ref)
    parity.check_codes(cu, cu_ref, ref["U"], su_ref, O.COL, group)
    parity.check_codes(cv, cv_ref, ref["V"], sv_ref, O.ROW, group)


def test_config5_vo_pair_full_oracle(env):
    """V 4608 x 2048 with O 4096 x 4608, 16 kv-head blocks of 128, two query heads per block, 4 bit:
    paired losses and gradient, then one Alg. 1 iteration, all against the full oracle."""
    torch, cafeq = env
    bits, group, k, rep = 4, 128, 128, 2
    ta, tb = WL.config5_tensor("v"), WL.config5_tensor("o")
    A, B = WL.bf16_bits_to_f32(ta["bits16"]), WL.bf16_bits_to_f32(tb["bits16"])
    T = WL.config5_transform("vo")
    P64 = O.block_inverse(T)
    P = P64.astype(np.float32)
    losses, grad, outs = cafeq.dual_proxy_loss_fwd_bwd(_dev_bf16(torch, ta["bits16"]), _dev_bf16(torch, tb["bits16"]),
                                                       _dev(torch, T), _dev(torch, P), bits, group, rep, 5.0,
                                                       True, True)
    torch.cuda.synchronize()
    losses = losses.cpu().numpy().astype(np.float64)
    ref = O.dual_lse(A, B, T, P, bits, group, rep, 5.0)
    for i, name in enumerate(("errU_sq", "errV_sq", "l2A_sq", "l2B_sq", "lse")):
        parity.check_scalar(losses[i], ref[name], what=name)
    parity.check_grad(grad.cpu().numpy(), ref["gradT"])
    cu, su, cv, sv = [x.cpu().numpy() for x in outs]
    cu_ref, su_ref, _ = O.rtn_sym(ref["U"], bits, group, O.COL)
    cv_ref, sv_ref, _ = O.rtn_sym(ref["V"], bits, group, O.ROW)
    parity.check_scales(su, su_ref)
    parity.check_scales(sv, sv_ref)
    parity.check_codes(cu, cu_ref, ref["U"], su_ref, O.COL, group)
    parity.check_codes(cv, cv_ref, ref["V"], sv_ref, O.ROW, group)

    # one iteration of Alg. 1 on the transformed pair (the oracle's U, V in float32), line by line
    U, V = ref["U"].astype(np.float32), ref["V"].astype(np.float32)
    cu0, su0, _ = O.rtn_sym(U, bits, group, O.COL)
    Uh = _dequant(cu0, su0, group, O.COL)
    _, _, Vt, Ut = O.adaptive_round_step(U, V, Uh, bits, group, k, rep, half=0)
    cv1, sv1, _ = O.rtn_sym(Vt, bits, group, O.ROW)
    cu1, su1, _ = O.rtn_sym(Ut, bits, group, O.COL)
    Ud, Vd = _dev(torch, U), _dev(torch, V)
    dcu, dsu = _dev(torch, cu0), _dev(torch, su0.astype(np.float32))
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros(sv1.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep, half=1)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsv.cpu().numpy(), sv1)
    parity.check_codes(dcv.cpu().numpy(), cv1, Vt, sv1, O.ROW, group)
    dcv2, dsv2 = _dev(torch, cv1), _dev(torch, sv1.astype(np.float32))
    dcu2 = torch.zeros(U.shape, dtype=torch.int8, device="cuda:0")
    dsu2 = torch.zeros(su1.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu2, dsu2, dcv2, dsv2, bits, group, k, rep, half=2)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsu2.cpu().numpy(), su1)
    parity.check_codes(dcu2.cpu().numpy(), cu1, Ut, su1, O.COL, group)


def test_config5_final_quantize_of_the_largest_matrix(env):
    """Plain RTN of the 170 M-element gate matrix (bfloat16), bit-exact on sampled rows, and the
    error sum against the float64 value recomputed from the device's own codes and scales."""
    torch, cafeq = env
    bits, group = 4, 128
    t = WL.config5_tensor("gate")
    codes, scales, err = cafeq.rtn_quantize(_dev_bf16(torch, t["bits16"]), bits, group, O.COL, want_err=True)
    torch.cuda.synchronize()
    rows = _sample(t["bits16"].shape[0], 252, 5301)
    Ws = WL.bf16_bits_to_f32(t["bits16"][rows])
    c_ref, s_ref, zq_ref = O.rtn_sym(Ws, bits, group, O.COL)
    rd = torch.from_numpy(rows).to("cuda:0")
    np.testing.assert_array_equal(codes[rd].cpu().numpy(), c_ref)
    np.testing.assert_array_equal(scales[rd].cpu().numpy(), s_ref.astype(np.float32))
    # error sum: float64 over row chunks from the device's codes and scales
    tot = 0.0
    cn, sn = codes.cpu().numpy(), scales.cpu().numpy()
    for r0 in range(0, cn.shape[0], 4096):
        w = WL.bf16_bits_to_f32(t["bits16"][r0:r0 + 4096]).astype(np.float64)
        tot += float(((_dequant(cn[r0:r0 + 4096], sn[r0:r0 + 4096], group, O.COL) - w) ** 2).sum())
    parity.check_scalar(float(err), tot, rel=1e-5, what="err_sq")
