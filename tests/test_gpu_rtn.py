"""GPU parity: cafeq_rtn_quantize against the oracle, bit-exact codes and scales."""
import numpy as np
import pytest

from oracle import cafeq_oracle as O
from paper_2511_19705_amd import workloads as WL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2511_19705_amd import cafeq
    return torch, cafeq


def _run(env, W_np, bits, group, axis, bf16=False, ld_pad=0):
    torch, cafeq = env
    dev = torch.device("cuda:0")
    if bf16:
        bits16 = WL.to_bf16_bits(W_np)
        W_ref = WL.bf16_bits_to_f32(bits16)
        Wd = torch.from_numpy(bits16.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        W_ref = W_np
        Wd = torch.from_numpy(W_np).to(dev)
    if ld_pad:
        big = torch.zeros((Wd.shape[0], Wd.shape[1] + ld_pad), dtype=Wd.dtype, device=dev)
        big[:, :Wd.shape[1]] = Wd
        Wd = big[:, :W_np.shape[1]]
    codes, scales, err = cafeq.rtn_quantize(Wd, bits, group, axis, want_err=True)
    torch.cuda.synchronize()
    c_ref, s_ref, zh = O.rtn_sym(W_ref, bits, group, axis)
    np.testing.assert_array_equal(codes.cpu().numpy(), c_ref)
    np.testing.assert_array_equal(scales.cpu().numpy(), s_ref.astype(np.float32))
    ref = float(((zh - W_ref.astype(np.float64)) ** 2).sum())
    assert abs(float(err.item()) - ref) <= 1e-5 * ref + 1e-30


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("group", [4, 32, 64, 128, 256, 0, 96])
def test_col_groups(env, bits, group):
    W = WL.student_t3((37, 768), 900 + bits)          # ragged: 37 rows, tail vector blocks
    WL.scale_random_columns(W, 2, 10.0, 5)
    _run(env, W, bits, group, O.COL)


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("group", [16, 32, 64, 128, 256, 0, 48, 8])
def test_row_groups(env, bits, group):
    W = WL.student_t3((768, 332), 910 + bits)         # 332 columns: ragged 256-column tiles
    _run(env, W, bits, group, O.ROW)


@pytest.mark.parametrize("axis,group", [(O.COL, 128), (O.ROW, 64), (O.COL, 0), (O.ROW, 40)])
def test_bf16_storage_and_padded_ld(env, axis, group):
    W = WL.student_t3((320, 512), 920)
    _run(env, W, 4, group, axis, bf16=True)
    _run(env, W, 3, group, axis, bf16=False, ld_pad=64)
    _run(env, W, 3, group, axis, bf16=True, ld_pad=64)


def test_zero_groups_and_outliers(env):
    W = WL.gaussian((64, 256), 930)
    W[3, :] = 0
    W[:, 128:160] = 0
    W[10, 7] = 1e30
    W[11, 9] = 1e-42          # denormal absmax inside an otherwise zero group
    W[11, :8] = 0
    W[11, 9:32] = 0
    _run(env, W, 4, 32, O.COL)
    _run(env, W, 4, 32, O.ROW)


def test_config1_and_config2_full_size(env):
    c1 = WL.config1()
    _run(env, c1["W"], 4, 32, O.COL)
    c2 = WL.config2()
    for bits in c2["bits"]:
        _run(env, c2["W"], bits, 128, O.COL)


def test_argument_errors(env):
    torch, cafeq = env
    W = torch.zeros((8, 30), device="cuda:0")
    with pytest.raises(cafeq.CafeqError):
        cafeq.rtn_quantize(W, 4, 32, O.COL)            # cols % 4 != 0 -> BAD_SHAPE
    W = torch.zeros((8, 64), device="cuda:0")
    with pytest.raises(cafeq.CafeqError):
        cafeq.rtn_quantize(W, 4, 48, O.COL)            # 64 % 48 != 0
    with pytest.raises(cafeq.CafeqError):
        cafeq.rtn_quantize(W, 9, 32, O.COL)            # bits out of range


# ---- the min/max grid of Eq. (1) ------------------------------------------------------------
def _run_minmax(env, W_np, bits, group, axis, bf16=False):
    torch, cafeq = env
    dev = torch.device("cuda:0")
    if bf16:
        bits16 = WL.to_bf16_bits(W_np)
        W_ref = WL.bf16_bits_to_f32(bits16)
        Wd = torch.from_numpy(bits16.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        W_ref = W_np
        Wd = torch.from_numpy(W_np).to(dev)
    codes, scales, mins, err = cafeq.rtn_quantize_minmax(Wd, bits, group, axis, want_err=True)
    torch.cuda.synchronize()
    c_ref, s_ref, lo_ref, zh = O.rtn_asym(W_ref, bits, group, axis, "f32")
    np.testing.assert_array_equal(codes.cpu().numpy().astype(np.int16), c_ref)
    np.testing.assert_array_equal(scales.cpu().numpy(), s_ref.astype(np.float32))
    np.testing.assert_array_equal(mins.cpu().numpy(), lo_ref.astype(np.float32))
    ref = float(((zh - W_ref.astype(np.float64)) ** 2).sum())
    assert abs(float(err.item()) - ref) <= 1e-5 * ref + 1e-30


@pytest.mark.parametrize("bits", [1, 3, 4, 8])
@pytest.mark.parametrize("group", [4, 64, 256, 0, 96])
def test_minmax_col_groups(env, bits, group):
    W = WL.student_t3((37, 768), 930 + bits)
    WL.scale_random_columns(W, 2, 10.0, 6)
    W[5, :96] = 0.25                                   # a constant group (and part of larger ones)
    _run_minmax(env, W, bits, group, O.COL)


@pytest.mark.parametrize("bits,group", [(4, 64), (3, 0), (4, 48)])
def test_minmax_row_groups_and_bf16(env, bits, group):
    W = WL.student_t3((768, 332), 940 + bits)
    _run_minmax(env, W, bits, group, O.ROW)
    _run_minmax(env, np.ascontiguousarray(W.T[:64]), bits, 128 if group else 0, O.COL, bf16=True)


def test_minmax_per_channel_on_the_2b_shaped_matrix(env):
    """Per-channel Eq. (1) (one group per output channel, the setting of the paper's tables) at the
    size of configuration 2, bit-exact."""
    c2 = WL.config2()
    _run_minmax(env, c2["W"], 4, 0, O.COL)
    _run_minmax(env, c2["W"], 4, 256, O.COL)
