"""cafeq_rtn_quantize_static (the entry point that allocates nothing) against cafeq_rtn_quantize,
through the C ABI, on two calls in a row -- the second on a smaller input, so that what the first
call left in the built-in scratch array would show if anything depended on it."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(cq, R, C, bits, group, axis, seed, dtype=torch.float32):
    g = torch.Generator(device="cpu").manual_seed(seed)
    W = (torch.randn((R, C), generator=g) * 0.02).to(dtype).cuda()
    ref_codes, ref_scales, ref_err = cq.rtn_quantize(W, bits, group, axis, want_err=True)
    codes = torch.full((R, C), 99, dtype=torch.int8, device="cuda")
    scales = torch.full(ref_scales.shape, -1.0, dtype=torch.float32, device="cuda")
    err = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    cq.rtn_quantize_static(W, codes, scales, err, bits, group, axis)
    torch.cuda.synchronize()
    # same kernels, same launch shape, same fixed-order reduction: everything is bit-identical
    assert torch.equal(codes, ref_codes)
    assert torch.equal(scales, ref_scales)
    assert torch.equal(err, ref_err)
    assert float(err) > 0


def test_static_scratch_matches_workspace_variant_on_two_calls_in_a_row():
    from paper_2511_19705_amd import cafeq as cq
    _case(cq, 1024, 4096, 4, 128, cq.AXIS_COL, 1)      # 4096 partials
    _case(cq, 96, 512, 3, 64, cq.AXIS_COL, 2)          # smaller: 48 partials, the rest of the array is stale
    _case(cq, 512, 768, 4, 64, cq.AXIS_ROW, 3)         # strided-axis kernel
    _case(cq, 64, 256, 4, 32, cq.AXIS_ROW, 4, torch.bfloat16)
    _case(cq, 40, 100, 4, 20, cq.AXIS_COL, 5)          # the any-length kernel


def test_static_scratch_rejects_inputs_beyond_its_limit_and_bad_arguments():
    from paper_2511_19705_amd import cafeq as cq
    import ctypes
    # 65537 * 1024 * 4 elements would need more partials than the built-in array holds: refused on the
    # host from the shape alone (the data pointer is never touched, so a small tensor stands in)
    W = torch.zeros((16, 16), dtype=torch.float32, device="cuda")
    m = cq.mat(W)
    m.rows, m.cols, m.ld = 65537 * 4, 1024, 1024
    cfg = cq.QuantCfg(4, 128, cq.AXIS_COL, 0)
    err = torch.zeros(1, device="cuda")
    rc = cq.lib.cafeq_rtn_quantize_static(ctypes.byref(m), ctypes.byref(cfg), cq._ptr(W), None, cq._ptr(err), None)
    assert rc == -7
    rc = cq.lib.cafeq_rtn_quantize_static(None, ctypes.byref(cfg), cq._ptr(W), None, None, None)
    assert rc == -1
