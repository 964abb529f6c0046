"""Shared comparison rules for the GPU parity tests (tolerances and why).

* integer outputs on the untransformed path: bit-exact.
* transformed path: the GPU forms Z with float32-level accuracy (exact three-way bfloat16
  operand split on the matrix cores, float32 accumulation), the oracle in float64 then
  rounds to float32; both decide the code with the same float32 recipe, so
  codes may differ only where Z sits within accumulation error of a rounding tie: at most
  1e-5 of the codes (at least one allowed on tiny inputs), each by exactly 1, each at a tie.
* where "a tie" is decided: by default |z/s - (n + 1/2)| < 2e-4; the main single-matrix and pair checks derive
  the bound per element from the arithmetic instead (tie_tolerance below): the transform's error on one element
  is a sum of k rounding errors of relative size `unit`, random in sign, so about unit * rss with rss the
  root-sum-square of the element's k terms; the group's scale moves with the error at its arg-max; eight
  standard deviations of the two together, in units of the scale, is the tolerance.
* Z itself: |err| <= k * 2^-24 * (|W| . |T|) elementwise (the standard dot-product bound).
* losses and gradients: 1e-4 relative (gradients: relative to the largest entry and in
  Frobenius norm), the float32 budget the workload statement gives.
"""
import numpy as np

CODE_FRAC = 1e-5
REL = 1e-4


# Relative rounding unit per term of the forward transform: two float16 parts per operand (22 of float32's 24
# bits, the weights' second part truncated) where the kernel takes them -- blocks of 128, groups up to 128,
# grids of up to 4 bits -- else three bfloat16 parts with the products below 2^-24 dropped and float32 accumulation.
UNIT_HALF = 2.0 ** -20
UNIT_FULL = 2.0 ** -23


def forward_unit(k, group_k, bits, minmax=False):
    return UNIT_HALF if (k == 128 and group_k <= 128 and bits <= 4 and not minmax) else UNIT_FULL


def tie_tolerance(W, X, axis, rep, z_ref, scales_ref, group, unit):
    """Per-element bound on |z/s (device) - z/s (oracle)| from the arithmetic of the transform Z = W.X / X.W:
    8 * unit * (rss(element) + rss(arg-max of its group)) / scale, rss = root-sum-square of the element's terms
    (computed with the oracle's own block-diagonal routine on the squared operands)."""
    from oracle import cafeq_oracle as O
    W = np.asarray(W, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    rss = np.sqrt(O.blockdiag_apply(W * W, X * X, axis, rep))
    g = group if group else (z_ref.shape[1] if axis == 0 else z_ref.shape[0])
    zg = O._to_groups(np.abs(z_ref), axis, g)
    rg = O._to_groups(rss, axis, g)
    star = rg[np.arange(zg.shape[0]), np.argmax(zg, axis=1)]
    rss_star = O._from_groups(np.repeat(star[:, None], g, axis=1), z_ref.shape, axis, g)
    s_el = np.repeat(np.asarray(scales_ref, dtype=np.float64), g, axis=1 if axis == 0 else 0)
    with np.errstate(divide="ignore", invalid="ignore"):
        tol = 8.0 * unit * (rss + rss_star) / s_el
    return np.where(s_el > 0, tol, np.inf)


def check_codes(codes_gpu, codes_ref, z_ref, scales_ref, axis, group, tie_tol=2e-4):
    """tie_tol: a number, or an array like z_ref (tie_tolerance)."""
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
        tol = tie_tol[diff] if isinstance(tie_tol, np.ndarray) else tie_tol
        assert np.all(np.abs(x - np.floor(x) - 0.5) < tol), "a differing code is not at a rounding tie"
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


def dual_argmax_flip_slack(A, B, T, P, ref, group, rep, t, tol=4e-6):
    """Entrywise slack for the LogSumExp gradient of a pair: the sub-gradient differentiates each group's absmax
    at its arg-max element, and where the two largest magnitudes of a group differ by less than the float32
    accuracy of the transformed weights (relative ``tol``) either element is a correct choice.  For every such
    group the gradient may move by  p_G * (e_j2 a^T - e_j1 a^T)  (member A; through -P^T . P^T for member B);
    the sum of the absolute values of those moves bounds what a different, equally valid choice changes.
    Returns (slack [nb][k][k], number of ambiguous groups)."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    nb, k, _ = P.shape
    lse = ref["lse"]
    slack_u = np.zeros((nb, k, k))
    slack_gp = np.zeros((nb, k, k))
    n_amb = 0
    U, V = ref["U"], ref["V"]
    d1, d3 = A.shape[0], B.shape[1]
    gu = group if group else U.shape[1]
    Ug = np.abs(U).reshape(d1, U.shape[1] // gu, gu)
    top = np.argsort(Ug, axis=2)[:, :, -2:]                               # second largest, largest
    a2 = np.take_along_axis(Ug, top[:, :, :1], 2)[:, :, 0]
    a1 = np.take_along_axis(Ug, top[:, :, 1:], 2)[:, :, 0]
    for i, gi in zip(*np.nonzero(a1 - a2 <= tol * a1)):
        n_amb += 1
        p = np.exp(t * (a1[i, gi] - lse))
        for j in top[i, gi]:
            ax = gi * gu + j
            b = ax // k
            slack_u[b, :, ax % k] += p * np.abs(A[i, b * k:(b + 1) * k])   # gradT_b[m][j] += p sign A[i][m]
    gv = group if group else V.shape[0]
    Vg = np.abs(V).reshape(V.shape[0] // gv, gv, d3)
    top = np.argsort(Vg, axis=1)[:, -2:, :]
    a2 = np.take_along_axis(Vg, top[:, :1, :], 1)[:, 0, :]
    a1 = np.take_along_axis(Vg, top[:, 1:, :], 1)[:, 0, :]
    for gi, c in zip(*np.nonzero(a1 - a2 <= tol * a1)):
        n_amb += 1
        p = np.exp(t * (a1[gi, c] - lse))
        for j in top[gi, :, c]:
            ax = gi * gv + j
            q = ax // k
            b = q // rep
            slack_gp[b, ax % k, :] += p * np.abs(B[q * k:(q + 1) * k, c])  # G_P[b][j][m] += p sign B[q k + m][c]
    aPt = np.abs(P).transpose(0, 2, 1)
    return slack_u + aPt @ slack_gp @ aPt, n_amb


def check_grad_with_slack(g_gpu, g_ref, slack, rel=REL):
    g_ref = np.asarray(g_ref, dtype=np.float64)
    err = np.abs(g_gpu.astype(np.float64) - g_ref)
    assert np.all(err <= rel * np.abs(g_ref).max() + slack), \
        "gradient max error %g vs scale %g (beyond the arg-max slack)" % (err.max(), np.abs(g_ref).max())
    assert np.linalg.norm(err) <= rel * np.linalg.norm(g_ref) + np.linalg.norm(slack)


def check_codes_minmax(codes_gpu, codes_ref, z_ref, scales_ref, mins_ref, axis, group, tie_tol=2e-4):
    """The same rule on the min/max grid of Eq. (1): codes count steps of the group's scale from its minimum."""
    diff = codes_gpu.astype(np.int32) != codes_ref.astype(np.int32)
    n_bad = int(diff.sum())
    allowed = max(1, int(np.ceil(CODE_FRAC * codes_ref.size)))
    assert n_bad <= allowed, "%d of %d codes differ (allowed %d)" % (n_bad, codes_ref.size, allowed)
    if n_bad:
        d = np.abs(codes_gpu.astype(np.int32) - codes_ref.astype(np.int32))[diff]
        assert d.max() == 1, "a code differs by more than one level"
        g = group if group else (z_ref.shape[1] if axis == 0 else z_ref.shape[0])
        s_el = np.repeat(scales_ref.astype(np.float64), g, axis=1 if axis == 0 else 0)
        lo_el = np.repeat(mins_ref.astype(np.float64), g, axis=1 if axis == 0 else 0)
        x = (z_ref[diff] - lo_el[diff]) / s_el[diff]
        tol = tie_tol[diff] if isinstance(tie_tol, np.ndarray) else tie_tol
        assert np.all(np.abs(x - np.floor(x) - 0.5) < tol), "a differing code is not at a rounding tie"
    print("codes differing from the oracle: %d of %d (%.2e)" % (n_bad, codes_ref.size, n_bad / codes_ref.size))
    return n_bad


def check_mins(m_gpu, m_ref, scales_ref, levels, rtol=5e-6):
    """Group minima are transformed values themselves: compared relative to the group's range."""
    rng = scales_ref.astype(np.float64) * levels
    assert np.all(np.abs(m_gpu.astype(np.float64) - m_ref) <= rtol * rng + 1e-30)
