"""GPU parity: cafeq_adaptive_round_step (Alg. 1) and cafeq_block_inverse against the oracle.

Each line of Alg. 1 is checked on inputs produced by the oracle, so that a handful of
tie-flipped codes from one line cannot leak into the other line's normal equations; the
chained call (half = 0) is then checked through the paired quantization error it reaches.
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


def _pair(rowsA, colsB, k, nb, rep, seed):
    """Transformed pair (U, V) in float32, built on the host from a seeded raw pair."""
    A, B, T = WL.small_pair(rowsA, nb * k, k, rep, seed, eps=0.05)
    B = np.ascontiguousarray(B[:, :colsB])
    P = O.block_inverse(T)
    U = O.blockdiag_apply(A, T, O.COL).astype(np.float32)
    V = O.blockdiag_apply(B, P, O.ROW, rep).astype(np.float32)
    return U, V


def _dequant(codes, scales, group, axis):
    return codes.astype(np.float64) * np.repeat(scales.astype(np.float64), group, axis=1 if axis == O.COL else 0)


# (the last two: contraction lengths that end 12 and 4 into a step of 16 of the Gram kernels for heads of 128 / 256,
# shared heads with blocks of 256)
@pytest.mark.parametrize("k,group,rep,bits,extra", [(64, 64, 2, 4, 0), (32, 32, 1, 3, 0), (128, 64, 2, 4, 0),
                                                    (256, 64, 1, 4, 0), (256, 64, 2, 4, 260), (128, 64, 1, 4, 268)])
def test_each_line_against_oracle(env, k, group, rep, bits, extra):
    torch, cafeq = env
    nb = 2
    # rows of U and columns of V: at least k (full rank), ragged against the 128-line macro-tile
    U, V = _pair((200 if k <= 128 else 328) + extra, (136 if k <= 128 else 296) + extra, k, nb, rep, 500 + k + extra)
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    Uh = _dequant(cu, su, group, O.COL)
    # oracle: line 3 then line 4
    Uh1, Vh1, Vt, Ut = O.adaptive_round_step(U, V, Uh, bits, group, k, rep, half=0)
    cv_ref, sv_ref, _ = O.rtn_sym(Vt, bits, group, O.ROW)
    cu_ref, su_ref, _ = O.rtn_sym(Ut, bits, group, O.COL)

    Ud, Vd = _dev(torch, U), _dev(torch, V)
    # line 3 on the device, from the oracle's (bit-identical) codes of U
    dcu, dsu = _dev(torch, cu), _dev(torch, su.astype(np.float32))
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros(sv_ref.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep, half=1)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsv.cpu().numpy(), sv_ref)
    parity.check_codes(dcv.cpu().numpy(), cv_ref, Vt, sv_ref, O.ROW, group)
    # line 4 on the device, from the oracle's codes of V
    dcv2, dsv2 = _dev(torch, cv_ref), _dev(torch, sv_ref.astype(np.float32))
    dcu2 = torch.zeros(U.shape, dtype=torch.int8, device="cuda:0")
    dsu2 = torch.zeros(su_ref.shape, dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu2, dsu2, dcv2, dsv2, bits, group, k, rep, half=2)
    torch.cuda.synchronize()
    assert int(st.abs().sum()) == 0
    parity.check_scales(dsu2.cpu().numpy(), su_ref)
    parity.check_codes(dcu2.cpu().numpy(), cu_ref, Ut, su_ref, O.COL, group)


def test_chained_iterations_reach_the_oracle_pqe(env):
    torch, cafeq = env
    k, group, rep, bits, nb = 64, 64, 2, 4, 2
    U, V = _pair(264, 200, k, nb, rep, 600)
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    Uh = _dequant(cu, su, group, O.COL)
    Vh0 = O.rtn_sym(V, bits, group, O.ROW)[2]
    p_indep, _ = O.pqe(U, V, Uh, Vh0, k, rep)
    Uh_o, Vh_o = Uh, None
    for _ in range(3):
        Uh_o, Vh_o, _, _ = O.adaptive_round_step(U, V, Uh_o, bits, group, k, rep)
    p_ref, _ = O.pqe(U, V, Uh_o, Vh_o, k, rep)

    Ud, Vd = _dev(torch, U), _dev(torch, V)
    dcu, dsu = _dev(torch, cu), _dev(torch, su.astype(np.float32))
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros((V.shape[0] // group, V.shape[1]), dtype=torch.float32, device="cuda:0")
    for _ in range(3):
        cafeq.adaptive_round_step(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep, half=0)
    torch.cuda.synchronize()
    Uh_g = _dequant(dcu.cpu().numpy(), dsu.cpu().numpy(), group, O.COL)
    Vh_g = _dequant(dcv.cpu().numpy(), dsv.cpu().numpy(), group, O.ROW)
    p_gpu, _ = O.pqe(U, V, Uh_g, Vh_g, k, rep)
    assert p_ref < 0.95 * p_indep              # the algorithm helps on this input
    assert abs(p_gpu - p_ref) <= 2e-3 * p_ref  # and the device lands on the same error level


# (heads of 256 take the block elimination on the matrix pipe: the two equal columns fall into one pivot block in
# the first case and into different panels, of one quantization group, in the second)
@pytest.mark.parametrize("k,group,rows,cols,dup", [(32, 32, 136, 72, (5, 3)), (256, 64, 328, 296, (5, 3)),
                                                   (256, 64, 328, 296, (60, 3))])
def test_rank_deficient_head_falls_back_to_plain_rounding(env, k, group, rows, cols, dup):
    torch, cafeq = env
    rep, bits, nb = 1, 4, 2
    U, V = _pair(rows, cols, k, nb, rep, 700)
    U[:, dup[0]] = U[:, dup[1]]                # head 0: two identical columns -> singular Gram
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    Ud, Vd = _dev(torch, U), _dev(torch, V)
    dcu, dsu = _dev(torch, cu), _dev(torch, su.astype(np.float32))
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros((V.shape[0] // group, V.shape[1]), dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep, half=1).cpu().numpy()
    assert st[0] == 1 and st[2] == 0
    c_plain, s_plain, _ = O.rtn_sym(V[:k], bits, group, O.ROW)
    np.testing.assert_array_equal(dcv.cpu().numpy()[:k], c_plain)
    np.testing.assert_array_equal(dsv.cpu().numpy()[:k // group], s_plain.astype(np.float32))


def test_fewer_rows_than_columns_is_flagged(env):
    # U_b is 40 x 64: its Gram matrix has rank <= 40, the normal equations do not apply
    torch, cafeq = env
    k, group, rep, bits, nb = 64, 64, 1, 4, 1
    U, V = _pair(40, 72, k, nb, rep, 710)
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    dcv = torch.zeros(V.shape, dtype=torch.int8, device="cuda:0")
    dsv = torch.zeros((V.shape[0] // group, V.shape[1]), dtype=torch.float32, device="cuda:0")
    st = cafeq.adaptive_round_step(_dev(torch, U), _dev(torch, V), _dev(torch, cu), _dev(torch, su.astype(np.float32)),
                                   dcv, dsv, bits, group, k, rep, half=1).cpu().numpy()
    assert st[0] == 1
    c_plain, _, _ = O.rtn_sym(V, bits, group, O.ROW)
    np.testing.assert_array_equal(dcv.cpu().numpy(), c_plain)


@pytest.mark.parametrize("k", [32, 64, 128, 256])
def test_block_inverse(env, k):
    torch, cafeq = env
    T = WL.perturbed_blocks(3, k, 800 + k, eps=0.3)
    T[1] = 0
    T[1, :, 0] = 1.0                            # block 1 is singular
    Tinv, rr, rc_, status = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    status = status.cpu().numpy()
    assert list(status) == [0, 1, 0]
    for b in (0, 2):
        ref = np.linalg.inv(T[b].astype(np.float64))
        np.testing.assert_allclose(Tinv[b].cpu().numpy(), ref, rtol=0, atol=2e-6 * np.abs(ref).max())
        rho_r = O.rho_from_inverse(ref[None], O.COL)
        rho_c = O.rho_from_inverse(ref[None], O.ROW)
        np.testing.assert_allclose(rr.cpu().numpy()[b * k:(b + 1) * k], rho_r, rtol=1e-5)
        np.testing.assert_allclose(rc_.cpu().numpy()[b * k:(b + 1) * k], rho_c, rtol=1e-5)


@pytest.mark.parametrize("k", [32, 128, 256])
@pytest.mark.parametrize("scale", [1e-4, 1.0, 3e3])
def test_block_inverse_general_matrices(env, k, scale):
    """Dense Gaussian blocks (condition number of order k, pivots far from 1, rows that need
    pivoting) at several magnitudes: the elimination pre-scales by a power of two, so the
    accuracy relative to the inverse's largest entry must not depend on the magnitude."""
    torch, cafeq = env
    rng = np.random.default_rng(900 + k)
    T = (rng.standard_normal((4, k, k)) * scale).astype(np.float32)
    T[2, 0, 0] = 0.0                            # a zero in the first pivot position
    Tinv, rr, rc_, status = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    assert list(status.cpu().numpy()) == [0, 0, 0, 0]
    for b in range(4):
        A = T[b].astype(np.float64)
        ref = np.linalg.inv(A)
        got = Tinv[b].cpu().numpy().astype(np.float64)
        # float32 output rounding plus conditioning: residual check against the identity
        res = np.abs(got @ A - np.eye(k)).max()
        assert res <= 2e-6 * np.linalg.cond(A), (b, res)
        np.testing.assert_allclose(got, ref, rtol=0, atol=4e-6 * np.abs(ref).max())
        np.testing.assert_allclose(rr.cpu().numpy()[b * k:(b + 1) * k], (ref ** 2).sum(1), rtol=2e-5)
        np.testing.assert_allclose(rc_.cpu().numpy()[b * k:(b + 1) * k], (ref ** 2).sum(0), rtol=2e-5)


def test_block_inverse_singular_block_is_zeroed(env):
    torch, cafeq = env
    T = WL.perturbed_blocks(2, 64, 77, eps=0.2)
    T[0, 5] = T[0, 9]                           # two equal rows
    Tinv, rr, rc_, status = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    assert list(status.cpu().numpy()) == [1, 0]
    assert float(Tinv[0].abs().max()) == 0.0
    assert float(rr[:64].abs().max()) == 0.0 and float(rc_[:64].abs().max()) == 0.0


def test_block_inverse_rejects_other_block_sizes(env):
    torch, cafeq = env
    T = np.stack([np.eye(48, dtype=np.float32)] * 2)
    with pytest.raises(Exception):
        cafeq.block_inverse(_dev(torch, T))


@pytest.mark.parametrize("k,group,rep,bits", [(32, 32, 1, 3), (64, 64, 2, 4), (128, 64, 2, 4), (256, 64, 1, 4)])
def test_paired_quantization_error_against_the_definition(env, k, group, rep, bits):
    """cafeq_pqe gets the paired quantization error from k x k Gram matrices; the oracle forms the
    d1 x d3 products of the definition.  Checked on independently rounded members and again on
    the codes of one iteration of Alg. 1."""
    torch, cafeq = env
    nb = 2
    U, V = _pair(200 if k <= 128 else 328, 136 if k <= 128 else 296, k, nb, rep, 1200 + k)
    cu, su, _ = O.rtn_sym(U, bits, group, O.COL)
    cv, sv, _ = O.rtn_sym(V, bits, group, O.ROW)
    Uh, Vh = _dequant(cu, su, group, O.COL), _dequant(cv, sv, group, O.ROW)
    p_abs, p_rel = O.pqe(U, V, Uh, Vh, k, rep)
    Ud, Vd = _dev(torch, U), _dev(torch, V)
    dcu, dsu = _dev(torch, cu), _dev(torch, su.astype(np.float32))
    dcv, dsv = _dev(torch, cv), _dev(torch, sv.astype(np.float32))
    out = cafeq.pqe(Ud, Vd, dcu, dsu, dcv, dsv, bits, group, k, rep).cpu().numpy().astype(np.float64)
    parity.check_scalar(out[0], p_abs ** 2, what="pqe_sq")
    parity.check_scalar(np.sqrt(out[0] / out[1]), p_rel, what="relative pqe")
    # after one iteration of Alg. 1 (the oracle's): a smaller error made of correlated roundings
    _, _, Vt, Ut = O.adaptive_round_step(U, V, Uh, bits, group, k, rep, half=0)
    cv1, sv1, _ = O.rtn_sym(Vt, bits, group, O.ROW)
    cu1, su1, _ = O.rtn_sym(Ut, bits, group, O.COL)
    p1_abs, _ = O.pqe(U, V, _dequant(cu1, su1, group, O.COL), _dequant(cv1, sv1, group, O.ROW), k, rep)
    out1 = cafeq.pqe(Ud, Vd, _dev(torch, cu1), _dev(torch, su1.astype(np.float32)), _dev(torch, cv1),
                     _dev(torch, sv1.astype(np.float32)), bits, group, k, rep).cpu().numpy().astype(np.float64)
    parity.check_scalar(out1[0], p1_abs ** 2, what="pqe_sq after Alg. 1")
    assert p1_abs < p_abs and out1[0] < out[0]


@pytest.mark.parametrize("k", [64, 128])
def test_block_inverse_of_rotations_and_of_their_neighbours(env, k):
    """Blocks that are rotations to float32 accuracy take the transposition path, every other block of
    the same call the elimination: exact rotations, rotations perturbed at 1e-7 .. 1e-2, a scaled
    rotation and a reflection, all to the accuracy of the elimination's float32 output."""
    torch, cafeq = env
    rng = np.random.default_rng(300 + k)
    H = WL.haar_blocks(8, k, 301 + k).astype(np.float64)
    T = H.copy()
    for b, eps in ((1, 1e-7), (2, 1e-6), (3, 1e-5), (4, 1e-3), (5, 1e-2)):
        T[b] += eps * rng.standard_normal((k, k))
    T[6] *= 1.0 + 1e-4                                        # unit directions, wrong length
    T[7][:, 0] *= -1.0                                        # a reflection is orthogonal too
    T = T.astype(np.float32)
    Tinv, rr, rc_, status = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    assert int(status.abs().sum()) == 0
    for b in range(8):
        ref = np.linalg.inv(T[b].astype(np.float64))
        got = Tinv[b].cpu().numpy().astype(np.float64)
        np.testing.assert_allclose(got, ref, rtol=0, atol=2e-6 * np.abs(ref).max(), err_msg="block %d" % b)
        np.testing.assert_allclose(rr.cpu().numpy()[b * k:(b + 1) * k], (ref ** 2).sum(1), rtol=1e-5)
        np.testing.assert_allclose(rc_.cpu().numpy()[b * k:(b + 1) * k], (ref ** 2).sum(0), rtol=1e-5)
    # exact rotations come back as the transpose, bit for bit
    for b in (0, 7):
        np.testing.assert_array_equal(Tinv[b].cpu().numpy(), T[b].T)


def test_block_inverse_256_near_rotations_and_far_blocks(env):
    """Blocks of 256: rotations, scaled rotations and their neighbours are inverted by Newton-Schulz rounds (accepted
    on the residual they reach), everything else of the same call by the elimination -- all to float32 rounding
    accuracy, with squared norms and status."""
    torch, cafeq = env
    k = 256
    rng = np.random.default_rng(2560)
    H = WL.haar_blocks(10, k, 2561).astype(np.float64)
    T = H.copy()
    T[1] += 1e-6 * rng.standard_normal((k, k))
    T[2] += (1e-3 / np.sqrt(k)) * rng.standard_normal((k, k))
    T[3] = T[3] @ (np.eye(k) + (0.05 / np.sqrt(k)) * rng.standard_normal((k, k)))     # a transform part-way through learning
    T[4] = T[4] @ (np.eye(k) + (0.3 / np.sqrt(k)) * rng.standard_normal((k, k)))      # too far for the rounds
    T[5] *= 37.5                                                                      # scaled rotations: any factor
    T[6] *= 2e-3
    T[7][:, 0] *= -1.0                                                                # reflection
    T[8] = rng.standard_normal((k, k))                                                # dense, nothing like a rotation
    T[9] = 0.0                                                                        # singular
    T = T.astype(np.float32)
    Tinv, rr, rc_, status = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    st = status.cpu().numpy()
    assert list(st[:9]) == [0] * 9 and st[9] == 1
    for b in range(9):
        ref = np.linalg.inv(T[b].astype(np.float64))
        got = Tinv[b].cpu().numpy().astype(np.float64)
        # float32 rounding of the result, amplified by the condition number for the dense block
        tol = (2e-6 if b != 8 else 2e-4) * np.abs(ref).max()
        np.testing.assert_allclose(got, ref, rtol=0, atol=tol, err_msg="block %d" % b)
        np.testing.assert_allclose(rr.cpu().numpy()[b * k:(b + 1) * k], (ref ** 2).sum(1), rtol=1e-4 if b == 8 else 1e-5)
        np.testing.assert_allclose(rc_.cpu().numpy()[b * k:(b + 1) * k], (ref ** 2).sum(0), rtol=1e-4 if b == 8 else 1e-5)
    assert float(Tinv[9].abs().max()) == 0.0
    # run-to-run identical
    Tinv2, _, _, _ = cafeq.block_inverse(_dev(torch, T), want_rho=True)
    torch.cuda.synchronize()
    assert torch.equal(Tinv, Tinv2)
