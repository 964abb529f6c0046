"""The C-ABI library loads and exports every symbol include/cafeq.h declares
(no compute calls here: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_19705_amd", "libcafeq.so")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cafeq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cafeq_[a-z_]+)\s*\(", text)))


def test_header_declares_the_five_hot_path_calls():
    syms = declared_symbols()
    for name in ("cafeq_rtn_quantize", "cafeq_apply_transform", "cafeq_proxy_loss_fwd_bwd",
                 "cafeq_dual_proxy_loss_fwd_bwd", "cafeq_adaptive_round_step"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__ as ge
        ge.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    lib.cafeq_strerror.restype = ctypes.c_char_p
    assert lib.cafeq_strerror(0) == b"ok"
    assert lib.cafeq_version() >= 100


def test_host_side_argument_validation_needs_no_gpu():
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    lib = ctypes.CDLL(LIB)
    lib.cafeq_rtn_quantize.restype = ctypes.c_int
    # NULL descriptors are rejected on the host before any launch
    rc = lib.cafeq_rtn_quantize(None, None, None, None, None, None, None)
    assert rc == -1


def test_argument_errors_of_every_entry_point_are_reported_before_any_launch():
    """NULL / malformed arguments come back as negative status codes from the host-side checks
    (no GPU needed, nothing is launched)."""
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    lib = ctypes.CDLL(LIB)

    class Mat(ctypes.Structure):
        _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                    ("ld", ctypes.c_int64), ("dtype", ctypes.c_int32), ("prepared", ctypes.c_void_p)]

    class Cfg(ctypes.Structure):
        _fields_ = [("bits", ctypes.c_int32), ("group", ctypes.c_int32), ("axis", ctypes.c_int32),
                    ("mode", ctypes.c_int32)]

    for name in ("cafeq_rtn_quantize", "cafeq_rtn_quantize_minmax", "cafeq_block_inverse", "cafeq_apply_transform",
                 "cafeq_proxy_loss_fwd_bwd", "cafeq_dual_proxy_loss_fwd_bwd", "cafeq_adaptive_round_step",
                 "cafeq_pqe", "cafeq_orth_penalty", "cafeq_sgd_update", "cafeq_adam_update",
                 "cafeq_optimize_single", "cafeq_optimize_pair"):
        getattr(lib, name).restype = ctypes.c_int
    vp = ctypes.c_void_p
    null = vp(0)
    fake = vp(4096)          # a non-null, 16-byte aligned address that is never dereferenced on these paths
    assert lib.cafeq_block_inverse(null, 64, 1, null, null, null, null, null, null) < 0
    lib.cafeq_block_inverse.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, vp, vp]
    assert lib.cafeq_block_inverse(fake, 48, 1, fake, null, null, null, fake, null) < 0      # unsupported block size
    assert lib.cafeq_block_inverse(fake, 64, 0, fake, null, null, null, fake, null) < 0      # no blocks
    assert lib.cafeq_block_inverse(fake, 64, 1, fake, null, null, null, null, null) < 0      # no workspace
    m = Mat(4096, 8, 100, 100, 0)                                                              # 100 columns
    cfg = Cfg(4, 32, 0, 0)                                                                     # groups of 32: 100 % 32 != 0
    lib.cafeq_rtn_quantize.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(Cfg), vp, vp, vp, vp, vp]
    assert lib.cafeq_rtn_quantize(ctypes.byref(m), ctypes.byref(cfg), fake, null, null, null, null) < 0
    bad_bits = Cfg(9, 0, 0, 0)
    assert lib.cafeq_rtn_quantize(ctypes.byref(m), ctypes.byref(bad_bits), fake, null, null, null, null) < 0
    lib.cafeq_rtn_quantize_minmax.argtypes = [ctypes.POINTER(Mat), ctypes.POINTER(Cfg), vp, vp, vp, vp, vp, vp]
    assert lib.cafeq_rtn_quantize_minmax(ctypes.byref(m), ctypes.byref(cfg), fake, null, null, null, null, null) < 0
    misaligned = Mat(4100, 8, 128, 128, 0)
    ok_cfg = Cfg(4, 32, 0, 0)
    assert lib.cafeq_rtn_quantize(ctypes.byref(misaligned), ctypes.byref(ok_cfg), fake, null, null, null, null) < 0
    lib.cafeq_orth_penalty.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_float, vp, vp, vp, vp]
    assert lib.cafeq_orth_penalty(fake, 64, 1, 0.1, null, null, fake, null) < 0               # nothing to compute
    assert lib.cafeq_orth_penalty(fake, 40, 1, 0.1, fake, null, fake, null) < 0               # unsupported block size
    lib.cafeq_sgd_update.argtypes = [vp, vp, ctypes.c_float, vp, ctypes.c_int64, vp]
    assert lib.cafeq_sgd_update(null, fake, 0.1, null, 16, null) < 0
    assert lib.cafeq_sgd_update(fake, fake, 0.1, null, 0, null) < 0
    lib.cafeq_adam_update.argtypes = [vp, vp, vp, vp, ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                      ctypes.c_double, ctypes.c_int64, vp]
    assert lib.cafeq_adam_update(fake, fake, fake, fake, 0, 1e-3, 0.9, 0.999, 1e-8, 16, null) < 0    # steps count from 1
    assert lib.cafeq_adam_update(fake, fake, fake, fake, 1, 1e-3, 1.0, 0.999, 1e-8, 16, null) < 0    # beta1 must be < 1
    class Xf(ctypes.Structure):
        _fields_ = [("T", vp), ("Tinv", vp), ("k", ctypes.c_int32), ("nb", ctypes.c_int32), ("rep", ctypes.c_int32)]

    i64 = ctypes.c_int64
    lib.cafeq_infer_single.restype = ctypes.c_int
    lib.cafeq_infer_single.argtypes = [vp, ctypes.c_int, i64, ctypes.POINTER(Xf), vp, vp, i64, i64, ctypes.c_int, vp,
                                       i64, vp, vp]
    assert lib.cafeq_infer_single(null, 1, 256, None, fake, fake, 8, 256, 32, fake, 8, null, null) == -1   # no X
    assert lib.cafeq_infer_single(fake, 1, 250, None, fake, fake, 8, 250, 0, fake, 8, null, null) == -2    # in % 16
    assert lib.cafeq_infer_single(fake, 1, 256, None, fake, fake, 8, 256, 24, fake, 8, null, null) == -2   # group % 16
    assert lib.cafeq_infer_single(fake, 1, 256, None, fake, fake, 8, 256, 32, fake, 4, null, null) == -2   # ldy < out
    xf = Xf(null, fake, 64, 3, 1)
    assert lib.cafeq_infer_single(fake, 1, 256, ctypes.byref(xf), fake, fake, 8, 256, 32, fake, 8, fake, null) == -2
    xf = Xf(null, fake, 64, 4, 1)
    assert lib.cafeq_infer_single(fake, 1, 256, ctypes.byref(xf), fake, fake, 8, 256, 32, fake, 8, null, null) == -7
    xf = Xf(null, fake, 48, 4, 1)
    assert lib.cafeq_infer_single(fake, 1, 192, ctypes.byref(xf), fake, fake, 8, 192, 32, fake, 8, fake, null) == -4
    lib.cafeq_infer_workspace_bytes.restype = ctypes.c_size_t
    lib.cafeq_infer_workspace_bytes.argtypes = [ctypes.c_int, i64]
    assert lib.cafeq_infer_workspace_bytes(3, 256) == 3 * 256 * 4
    assert lib.cafeq_infer_workspace_bytes(0, 256) == 0
    lib.cafeq_strerror.restype = ctypes.c_char_p
    for code in range(-8, 1):
        assert len(lib.cafeq_strerror(code)) > 0
