"""Shared comparison rules for the GPU parity tests (tolerances and why).

* integer outputs on the untransformed path: bit-exact.
* transformed path: the GPU forms Z with float32-level accuracy (exact three-way bfloat16
  operand split on the matrix cores, float32 accumulation), the oracle in float64 then
  rounds to float32; both decide the code with the same float32 recipe, so
  codes may differ only where Z sits within accumulation error of a rounding tie: at most
  1e-5 of the codes (at least one allowed on tiny inputs), each by exactly 1, each at a tie.
* Z itself: |err| <= k * 2^-24 * (|W| . |T|) elementwise (the standard dot-product bound).
* losses and gradients: 1e-4 relative (gradients: relative to the largest entry and in
  Frobenius norm), the float32 budget the workload statement gives.
"""
import numpy as np

CODE_FRAC = 1e-5
REL = 1e-4


def check_codes(codes_gpu, codes_ref, z_ref, scales_ref, axis, group, tie_tol=2e-4):
    diff = codes_gpu != codes_ref
    n_bad = int(diff.sum())
    allowed = max(1, int(np.ceil(CODE_FRAC * codes_ref.size)))
    assert n_bad <= allowed, "%d of %d codes differ (allowed %d)" % (n_bad, codes_ref.size, allowed)
    if n_bad:
        d = np.abs(codes_gpu.astype(np.int32) - codes_ref.astype(np.int32))[diff]
        assert d.max() == 1, "a code differs by more than one level"
        g = group if group else (z_ref.shape[1] if axis == 0 else z_ref.shape[0])
        s_el = np.repeat(scales_ref.astype(np.float64), g, axis=1 if axis == 0 else 0)
        x = np.abs(z_ref[diff] / s_el[diff])
        assert np.all(np.abs(x - np.floor(x) - 0.5) < tie_tol), "a differing code is not at a rounding tie"
    print("codes differing from the oracle: %d of %d (%.2e)" % (n_bad, codes_ref.size, n_bad / codes_ref.size))
    return n_bad


def check_scales(s_gpu, s_ref, rtol=5e-6):
    np.testing.assert_allclose(s_gpu, s_ref, rtol=rtol, atol=0)


def check_scalar(got, ref, rel=REL, what=""):
    assert abs(got - ref) <= rel * abs(ref) + 1e-30, "%s: got %r, oracle %r" % (what, got, ref)


def check_grad(g_gpu, g_ref, rel=REL):
    g_ref = np.asarray(g_ref, dtype=np.float64)
    err = np.abs(g_gpu.astype(np.float64) - g_ref)
    assert err.max() <= rel * np.abs(g_ref).max(), "gradient max error %g vs scale %g" % (err.max(), np.abs(g_ref).max())
    assert np.linalg.norm(err) <= rel * np.linalg.norm(g_ref)
