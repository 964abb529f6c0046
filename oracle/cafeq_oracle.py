"""CPU oracle for the CafeQ hot path -- TEST INFRASTRUCTURE, not the product.

A plain, slow, NumPy float64 implementation of what the paper defines, written
from the paper and sharing no code with the HIP library.  Only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import it; the product
path never does.

What each function follows (section / equation of the CafeQ paper):

* ``rtn_asym``           -- Eq. (1) (uniform min/max quantizer), error bound Eq. (2).
* ``rtn_sym``            -- the symmetric absmax b-bit grid with codes in
                            [-2^(b-1), 2^(b-1)-1] (the quantizer of the workloads;
                            same rounding rule as Eq. (1): nearest integer).
* ``blockdiag_apply``    -- block-diagonal transform, Sec. 4.1 (single matrix) and
                            Sec. 4.2 (pair: U = W1 M, V = M^-1 W2).
* ``proxy_l2``           -- the l2 proxy  ||M^-1 Q(M W) - W||_F  (Sec. 4, inequality
                            after "Our approach for learning M").
* ``surrogate``          -- the stochastic-rounding upper bound that gradient descent
                            runs on (last line of the display ending Sec. 4.1's
                            "Optimization of M"), generalised to arbitrary groups,
                            and its gradient w.r.t. the transform blocks.
* ``surrogate_printed``  -- that same display evaluated literally as printed
                            (one group per contraction index, spanning the output dim).
* ``dual_lse``           -- LogSumExp surrogate of Sec. 4.2 and its gradient.
* ``pinv``, ``adaptive_round_step``, ``pqe`` -- Algorithm 1 (Sec. 5) and the paired
                            quantization error of Sec. 4.2.
* ``adaptive_bruteforce_column`` -- exhaustive up/down search used only as a pin.
* ``hadamard_matrix``, ``hadamard_apply``, ``hadamard_baseline`` -- the paper's "random" comparison
                            (caption of the block-size table in Sec. 4.1): a block-diagonal transform whose
                            blocks are randomized Hadamard matrices, then the same quantizer.
* ``dequantize``, ``infer_single`` -- the inference side of a single transformed matrix (Sec. 4.1, the
                            display Y^ = X M^-1 Q(MW)): the activations take the inverse transform, then the
                            product with the dequantized transformed weight.
* ``orth_penalty``       -- the orthonormality regulariser ||T T^T - I||_F / sqrt(d) of the
                            appendix on paired-quantization hyperparameters ("Constraints on T").
* ``sgd_step``, ``adam_step``, ``optimize_single``, ``optimize_pair`` -- the learning
                            procedure: gradient descent on the surrogate for a single matrix
                            (Sec. 4.1, "perform gradient descent with [the bound] as the loss"),
                            Adam on the LogSumExp surrogate for a pair (Sec. 4.2 and the same
                            appendix), the inverse recomputed every step.

Pinned by tests/test_oracle_*.py against: the paper's 2x2 toy example, Eq. (2),
closed forms (orthogonal transform, identity transform), central finite
differences, brute force on tiny inputs, the Moore-Penrose identities and naive
triple loops.  Not pinned ("parity unpinned"): the magnitudes of the relative l2
losses the paper's tables print, which need the real Gemma-2 weights.

Layout conventions: a weight is ``W[R][C]``; a transform is ``T[nb][k][k]`` with
inverse ``P[nb][k][k]``; axis COL (0): ``Z = W . blockdiag(T)`` (nb*k == C);
axis ROW (1): ``Z = blockdiag(T) . W`` where row-block ``q`` (k rows) uses block
``q // rep``.  Quantization groups are ``g`` consecutive elements along the same
axis (``g == 0``: the whole line; ``g == -1``: the whole tensor).
Scale arrays: axis COL -> ``[R][C/g]``; axis ROW -> ``[R/g][C]``.
"""
from __future__ import annotations

import itertools

import numpy as np

COL = 0
ROW = 1
SYM = 0
ASYM = 1


# ----------------------------------------------------------------------------
# group bookkeeping (pure indexing)
# ----------------------------------------------------------------------------
def _to_groups(Z, axis, g):
    """Return a 2-D array whose rows are the quantization groups of ``Z``."""
    R, C = Z.shape
    if g == -1:
        return Z.reshape(1, R * C)
    if axis == COL:
        g = C if g == 0 else g
        assert C % g == 0
        return Z.reshape(R * (C // g), g)
    g = R if g == 0 else g
    assert R % g == 0
    return np.ascontiguousarray(Z.T).reshape(C * (R // g), g)


def _from_groups(Xg, shape, axis, g):
    """Inverse of ``_to_groups`` for an array with one value per element."""
    R, C = shape
    if g == -1 or axis == COL:
        return Xg.reshape(R, C)
    return np.ascontiguousarray(Xg.reshape(C, R).T)


def _group_values_layout(vals, shape, axis, g):
    """One value per group -> the documented scale layout."""
    R, C = shape
    if g == -1:
        return vals.reshape(1, 1)
    if axis == COL:
        g = C if g == 0 else g
        return vals.reshape(R, C // g)
    g = R if g == 0 else g
    return np.ascontiguousarray(vals.reshape(C, R // g).T)


# ----------------------------------------------------------------------------
# quantizers
# ----------------------------------------------------------------------------
def rtn_sym(Z, bits, group, axis, arith="f32"):
    """Symmetric absmax round-to-nearest.

    Per group: a = max|z|, s = a / qmax, q = clamp(nearest_int(z / s), qmin, qmax),
    zhat = q * s, with qmax = 2^(b-1) - 1, qmin = -2^(b-1); ties to even.
    ``arith="f64"`` evaluates exactly that in float64.  ``arith="f32"`` is the
    single-precision realisation both sides agree on for deciding the integer:
    z is rounded to float32, inv = min(fl(qmax / a), FLT_MAX), q = nearest_int(fl(z * inv)),
    s = fl(a / qmax), zhat = fl(q * s).  An all-zero group gives s = 0, q = 0.

    Returns (codes int8 [R][C], scales [groups layout], zhat [R][C] float64).
    """
    qmax = 2 ** (bits - 1) - 1
    qmin = -(2 ** (bits - 1))
    ft = np.float32 if arith == "f32" else np.float64
    Zg = _to_groups(np.asarray(Z, dtype=np.float64), axis, group).astype(ft)
    a = np.max(np.abs(Zg), axis=1)                      # [groups]
    safe = np.where(a > 0, a, ft(1))
    if arith == "f32":
        with np.errstate(over="ignore"):
            # capped so that a denormal absmax cannot produce inf (and 0 * inf = nan)
            inv = np.minimum((ft(qmax) / safe).astype(ft), np.finfo(np.float32).max)
        x = (Zg * inv[:, None]).astype(ft)
    else:
        x = Zg / (safe / qmax)[:, None]
    q = np.clip(np.rint(x), qmin, qmax)
    q = np.where((a > 0)[:, None], q, 0.0)
    s = np.where(a > 0, (a / ft(qmax)).astype(ft), ft(0))
    zhat = (q.astype(ft) * s[:, None]).astype(ft)
    shape = np.shape(Z)
    codes = _from_groups(q, shape, axis, group).astype(np.int8)
    return (codes, _group_values_layout(s, shape, axis, group),
            _from_groups(zhat.astype(np.float64), shape, axis, group))


def rtn_asym(Z, bits, group, axis, arith="f64"):
    """Eq. (1): s = (max - min)/(2^b - 1), q = nearest_int((z - min)/s) in
    [0, 2^b - 1], zhat = s*q + min; a constant group gives q = 0, zhat = min.
    ``arith="f64"`` evaluates exactly that in float64.  ``arith="f32"`` is the
    single-precision realisation both sides agree on for deciding the integer (same pattern as
    ``rtn_sym``): z rounded to float32, r = fl(max - min), inv = min(fl((2^b-1) / r), FLT_MAX),
    q = nearest_int(fl(fl(z - min) * inv)), s = fl(r / (2^b-1)), zhat = fl(fl(q * s) + min).
    Returns (codes, scales, zeros(min), zhat)."""
    levels = 2 ** bits - 1
    ft = np.float32 if arith == "f32" else np.float64
    Zg = _to_groups(np.asarray(Z, dtype=np.float64), axis, group).astype(ft)
    lo = Zg.min(axis=1)
    hi = Zg.max(axis=1)
    rng = (hi - lo).astype(ft)
    s = (rng / ft(levels)).astype(ft)
    safe = np.where(rng > 0, rng, ft(1))
    if arith == "f32":
        with np.errstate(over="ignore"):
            inv = np.minimum((ft(levels) / safe).astype(ft), np.finfo(np.float32).max)
        x = ((Zg - lo[:, None]).astype(ft) * inv[:, None]).astype(ft)
    else:
        x = (Zg - lo[:, None]) / (safe / levels)[:, None]
    q = np.clip(np.rint(x), 0, levels)
    q = np.where((rng > 0)[:, None], q, 0.0)
    zhat = ((q.astype(ft) * s[:, None]).astype(ft) + lo[:, None]).astype(ft)
    shape = np.shape(Z)
    return (_from_groups(q, shape, axis, group).astype(np.int16),
            _group_values_layout(s, shape, axis, group),
            _group_values_layout(lo, shape, axis, group),
            _from_groups(zhat.astype(np.float64), shape, axis, group))


def quantize(Z, bits, group, axis, mode=SYM, arith="f32"):
    """zhat only, for either grid."""
    if mode == SYM:
        return rtn_sym(Z, bits, group, axis, arith)[2]
    return rtn_asym(Z, bits, group, axis, arith)[3]


# ----------------------------------------------------------------------------
# block-diagonal transform
# ----------------------------------------------------------------------------
def blockdiag_apply(W, X, axis, rep=1):
    """COL: Z[:, b] = W[:, b] @ X[b];  ROW: Z[q] = X[q // rep] @ W[q]  (k-row blocks)."""
    W = np.asarray(W, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    nb, k, _ = X.shape
    R, C = W.shape
    if axis == COL:
        assert rep == 1 and C == nb * k
        Wb = W.reshape(R, nb, k).transpose(1, 0, 2)          # [nb][R][k]
        return np.ascontiguousarray((Wb @ X).transpose(1, 0, 2)).reshape(R, C)
    assert R == nb * rep * k
    Wb = W.reshape(nb, rep, k, C)
    return (X[:, None, :, :] @ Wb).reshape(R, C)


def block_inverse(T):
    return np.linalg.inv(np.asarray(T, dtype=np.float64))


def rho_from_inverse(P, axis):
    """rho_j = sum_i (M^-1)_{ij}^2 in the paper's orientation.  With the row-major
    [out][in] weights used here: axis COL -> squared row norms of P, axis ROW ->
    squared column norms of P.  Shape [nb*k]."""
    P = np.asarray(P, dtype=np.float64)
    return (P ** 2).sum(axis=2 if axis == COL else 1).reshape(-1)


# ----------------------------------------------------------------------------
# l2 proxy (forward only)
# ----------------------------------------------------------------------------
def proxy_l2(W, T, P, bits, group, axis, rep=1, mode=SYM, arith="f32"):
    """Returns dict(l2_sq=||Q(Z) P - W||_F^2, err_z_sq=||Q(Z)-Z||_F^2, w_sq=||W||_F^2,
    Z, Zhat) with Z = transform(W, T)."""
    W = np.asarray(W, dtype=np.float64)
    Z = blockdiag_apply(W, T, axis, rep)
    Zhat = quantize(Z, bits, group, axis, mode, arith)
    E = Zhat - Z
    D = blockdiag_apply(E, P, axis, rep)
    return dict(l2_sq=float((D * D).sum()), err_z_sq=float((E * E).sum()),
                w_sq=float((W * W).sum()), Z=Z, Zhat=Zhat)


# ----------------------------------------------------------------------------
# stochastic-rounding surrogate and its gradient
# ----------------------------------------------------------------------------
def beta_const(bits, mode):
    """Per-element variance bound of stochastic rounding divided by (group absmax)^2.
    SYM: step s = a/qmax, variance <= s^2/4.  ASYM: range R <= 2a, variance
    <= R^2 / (4 (2^b-1)^2) <= a^2/(2^b-1)^2 (the constant the paper prints)."""
    if mode == SYM:
        qmax = 2 ** (bits - 1) - 1
        return 1.0 / (4.0 * qmax * qmax)
    return 1.0 / float((2 ** bits - 1) ** 2)


def _rho_lines(rho, nb, k, shape, axis, rep):
    R, C = shape
    if axis == COL:
        return np.broadcast_to(rho.reshape(1, C), (R, C))
    per_row = np.repeat(rho.reshape(nb, 1, k), rep, axis=1).reshape(R)
    return np.broadcast_to(per_row[:, None], (R, C))


def surrogate(W, T, P, bits, group, axis, rep=1, mode=SYM, group_axis=None,
              want_grad=True):
    """L_sur = beta * sum_elements rho_{j(e)} * a_{G(e)}^2, and dL/dT.

    ``rho_j`` is the squared norm of the slice of the inverse transform that
    multiplies the error at transformed-axis index j; ``a_G`` is the absmax of
    the element's quantization group in Z = transform(W, T).  ``group_axis``
    defaults to ``axis`` (groups run along the transformed axis).

    Gradient (T only; P is a function of T): through Z with the absmax treated
    as |Z| at the arg-max element (lowest flat index on ties), and through
    rho(P) with dP = -P dT P.
    """
    W = np.asarray(W, dtype=np.float64)
    T = np.asarray(T, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    nb, k, _ = T.shape
    gax = axis if group_axis is None else group_axis
    beta = beta_const(bits, mode)
    Z = blockdiag_apply(W, T, axis, rep)
    rho = rho_from_inverse(P, axis)
    rho_e = _rho_lines(rho, nb, k, W.shape, axis, rep)

    Zg = _to_groups(Z, gax, group)
    rg = _to_groups(np.ascontiguousarray(rho_e), gax, group).sum(axis=1)   # sum_{e in G} rho
    amax_idx = np.argmax(np.abs(Zg), axis=1)                              # first max
    rows = np.arange(Zg.shape[0])
    zstar = Zg[rows, amax_idx]
    a = np.abs(zstar)
    loss = float(beta * (a * a * rg).sum())
    if not want_grad:
        return loss, None

    # dL/dZ: one non-zero per group
    Sg = np.zeros_like(Zg)
    Sg[rows, amax_idx] = 2.0 * beta * rg * zstar
    S = _from_groups(Sg, W.shape, gax, group)
    # v_j = beta * sum over elements with transformed-axis index j of a_G(e)^2
    a2_e = _from_groups(np.repeat((a * a)[:, None], Zg.shape[1], axis=1), W.shape, gax, group)
    R, C = W.shape
    if axis == COL:
        v = beta * a2_e.sum(axis=0)                                       # [C] = [nb*k]
        v = v.reshape(nb, k)
        Wb = W.reshape(R, nb, k).transpose(1, 2, 0)                       # [nb][k][R]  (W_b^T)
        Sb = S.reshape(R, nb, k).transpose(1, 0, 2)                       # [nb][R][k]
        g_z = Wb @ Sb
        Pt = P.transpose(0, 2, 1)
        g_p = -2.0 * (Pt @ (v[:, :, None] * P) @ Pt)
    else:
        v_rows = beta * a2_e.sum(axis=1)                                  # [R]
        v = v_rows.reshape(nb, rep, k).sum(axis=1)                        # [nb][k]
        Sb = S.reshape(nb, rep, k, C)
        Wb = W.reshape(nb, rep, k, C)
        g_z = (Sb @ Wb.transpose(0, 1, 3, 2)).sum(axis=1)                 # sum_q S_q W_q^T
        Pt = P.transpose(0, 2, 1)
        g_p = -2.0 * (Pt @ (P * v[:, None, :]) @ Pt)
    return loss, g_z + g_p


def surrogate_printed(W_in_out, M, bits):
    """The bound exactly as the paper prints it, for a weight in the paper's own
    orientation (``W_in_out`` is d1 x d2, y = x W; M is dense d1 x d1):
        d2 / (2^N - 1)^2 * sum_i sum_j (M^-1)_{ij}^2 * ||(M W)_j||_inf^2
    evaluated with explicit loops."""
    W = np.asarray(W_in_out, dtype=np.float64)
    M = np.asarray(M, dtype=np.float64)
    d1, d2 = W.shape
    Minv = np.linalg.inv(M)
    MW = M @ W
    total = 0.0
    for i in range(d1):
        for j in range(d1):
            total += Minv[i, j] ** 2 * np.max(np.abs(MW[j, :])) ** 2
    return d2 / float((2 ** bits - 1) ** 2) * total


# ----------------------------------------------------------------------------
# paired transform: forward errors, LogSumExp surrogate and gradient
# ----------------------------------------------------------------------------
def dual_lse(A, B, T, P, bits, group, rep=1, t=5.0, arith="f32", want_grad=True, mode=SYM):
    """Member A [d1 x nb*k] gets T on its columns (U = A T); member B
    [nb*rep*k x d3] gets P = T^-1 on its rows (V = P B).

    Returns dict with
      errU_sq, errV_sq : ||Q(U)-U||_F^2, ||Q(V)-V||_F^2
      l2A_sq, l2B_sq   : ||Q(U) P - A||_F^2, ||T Q(V) - B||_F^2
      lse              : (1/t) log( sum over every group of U and of V of exp(t * absmax) )
      n_groups, gradT  : d lse / dT  (through U directly, through V via dP = -P dT P)
    One LSE term per quantization group; with group = whole channel this is the
    paper's sum over m_u(i) and m_v(j).  ``mode`` selects the grid Q rounds to (the symmetric
    one or Eq. (1)); the LogSumExp is a function of the group maxima alone and does not depend on it."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    T = np.asarray(T, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    nb, k, _ = T.shape
    U = blockdiag_apply(A, T, COL)
    V = blockdiag_apply(B, P, ROW, rep)
    Uh = quantize(U, bits, group, COL, mode, arith)
    Vh = quantize(V, bits, group, ROW, mode, arith)
    EU = Uh - U
    EV = Vh - V
    DA = blockdiag_apply(EU, P, COL)
    DB = blockdiag_apply(EV, T, ROW, rep)

    Ug = _to_groups(U, COL, group)
    Vg = _to_groups(V, ROW, group)
    iu = np.argmax(np.abs(Ug), axis=1)
    iv = np.argmax(np.abs(Vg), axis=1)
    ru = np.arange(Ug.shape[0])
    rv = np.arange(Vg.shape[0])
    au = np.abs(Ug[ru, iu])
    av = np.abs(Vg[rv, iv])
    allmax = np.concatenate([au, av])
    mstar = allmax.max()
    sumexp = np.exp(t * (allmax - mstar)).sum()
    lse = mstar + np.log(sumexp) / t
    out = dict(errU_sq=float((EU * EU).sum()), errV_sq=float((EV * EV).sum()),
               l2A_sq=float((DA * DA).sum()), l2B_sq=float((DB * DB).sum()),
               lse=float(lse), n_groups=int(allmax.size), U=U, V=V, Uh=Uh, Vh=Vh)
    if not want_grad:
        return out
    pu = np.exp(t * (au - mstar)) / sumexp
    pv = np.exp(t * (av - mstar)) / sumexp
    SUg = np.zeros_like(Ug)
    SUg[ru, iu] = pu * np.sign(Ug[ru, iu])
    SVg = np.zeros_like(Vg)
    SVg[rv, iv] = pv * np.sign(Vg[rv, iv])
    SU = _from_groups(SUg, U.shape, COL, group)
    SV = _from_groups(SVg, V.shape, ROW, group)
    d1 = A.shape[0]
    d3 = B.shape[1]
    g_u = A.reshape(d1, nb, k).transpose(1, 2, 0) @ SU.reshape(d1, nb, k).transpose(1, 0, 2)
    GP = (SV.reshape(nb, rep, k, d3) @ B.reshape(nb, rep, k, d3).transpose(0, 1, 3, 2)).sum(axis=1)
    Pt = P.transpose(0, 2, 1)
    g_v = -(Pt @ GP @ Pt)
    out["gradT"] = g_u + g_v
    return out


# ----------------------------------------------------------------------------
# Algorithm 1: adaptive rounding on a coupled pair
# ----------------------------------------------------------------------------
def pinv(M):
    """Moore-Penrose pseudoinverse through the SVD; singular values below
    max(shape) * eps * sigma_max are treated as zero."""
    M = np.asarray(M, dtype=np.float64)
    u, s, vt = np.linalg.svd(M, full_matrices=False)
    cut = max(M.shape) * np.finfo(np.float64).eps * (s[0] if s.size else 0.0)
    sinv = np.where(s > cut, 1.0 / np.where(s > cut, s, 1.0), 0.0)
    return (vt.T * sinv[None, :]) @ u.T


def adaptive_targets_V(U, Uh, V, k, rep):
    """Line 3 of Algorithm 1 per head: V'_q = pinv(Uh_b) U_b V_q, b = q // rep."""
    U = np.asarray(U, dtype=np.float64)
    Uh = np.asarray(Uh, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    nb = U.shape[1] // k
    out = np.empty_like(V)
    for b in range(nb):
        Ab = pinv(Uh[:, b * k:(b + 1) * k]) @ U[:, b * k:(b + 1) * k]     # k x k
        for q in range(b * rep, (b + 1) * rep):
            out[q * k:(q + 1) * k, :] = Ab @ V[q * k:(q + 1) * k, :]
    return out


def adaptive_targets_U(U, V, Vh, k, rep):
    """Line 4 of Algorithm 1 per head: U'_b = U_b V_[b] pinv(Vh_[b]) where V_[b]
    places the rep row-blocks of head b side by side (k x rep*d3)."""
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Vh = np.asarray(Vh, dtype=np.float64)
    nb = U.shape[1] // k
    out = np.empty_like(U)
    for b in range(nb):
        Vs = np.concatenate([V[q * k:(q + 1) * k, :] for q in range(b * rep, (b + 1) * rep)], axis=1)
        Vhs = np.concatenate([Vh[q * k:(q + 1) * k, :] for q in range(b * rep, (b + 1) * rep)], axis=1)
        Bb = Vs @ pinv(Vhs)                                                # k x k
        out[:, b * k:(b + 1) * k] = U[:, b * k:(b + 1) * k] @ Bb
    return out


def adaptive_round_step(U, V, Uh, bits, group, k, rep=1, half=0, Vh=None,
                        mode=SYM, arith="f32"):
    """One iteration of Algorithm 1 in transformed coordinates (W1 := U, W2 := V),
    every Q() recomputing its own group scales.  half=0: lines 3 and 4; half=1:
    line 3 only; half=2: line 4 only (needs Vh).  Groups of U run along its
    columns (axis COL), groups of V along its rows (axis ROW).
    Returns (Uh_new, Vh_new, V_target, U_target)."""
    Vt = Ut = None
    if half in (0, 1):
        Vt = adaptive_targets_V(U, Uh, V, k, rep)
        Vh = quantize(Vt, bits, group, ROW, mode, arith)
    if half in (0, 2):
        Ut = adaptive_targets_U(U, V, Vh, k, rep)
        Uh = quantize(Ut, bits, group, COL, mode, arith)
    return Uh, Vh, Vt, Ut


def pqe(U, V, Uh, Vh, k, rep=1):
    """Paired quantization error over heads: sqrt(sum_q ||Uh_b Vh_q - U_b V_q||_F^2),
    b = q // rep, and the same relative to sqrt(sum_q ||U_b V_q||_F^2)."""
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    nq = V.shape[0] // k
    num = den = 0.0
    for q in range(nq):
        b = q // rep
        ref = U[:, b * k:(b + 1) * k] @ V[q * k:(q + 1) * k, :]
        got = np.asarray(Uh, dtype=np.float64)[:, b * k:(b + 1) * k] @ \
            np.asarray(Vh, dtype=np.float64)[q * k:(q + 1) * k, :]
        num += ((got - ref) ** 2).sum()
        den += (ref ** 2).sum()
    return float(np.sqrt(num)), float(np.sqrt(num / den)) if den > 0 else 0.0


def adaptive_bruteforce_column(Uh_b, target_prod_col, vt_col, bits, group):
    """Pin for line 3: for one column of one head, with the group scales fixed to
    those the step derives from its own target ``vt_col`` (length k), enumerate
    every floor/ceil choice of vt/s per element and return the dequantized column
    minimising ||Uh_b (s*q) - target_prod_col||^2 together with that minimum.
    Exponential in k: tiny inputs only."""
    k = vt_col.size
    g = k if group == 0 else group
    qmax = 2 ** (bits - 1) - 1
    qmin = -(2 ** (bits - 1))
    s = np.empty(k)
    for g0 in range(0, k, g):
        s[g0:g0 + g] = np.max(np.abs(vt_col[g0:g0 + g])) / qmax
    safe = np.where(s > 0, s, 1.0)
    lo = np.floor(vt_col / safe)
    best = None
    best_val = np.inf
    for choice in itertools.product((0.0, 1.0), repeat=k):
        q = np.clip(lo + np.array(choice), qmin, qmax)
        cand = q * s
        val = float(((Uh_b @ cand - target_prod_col) ** 2).sum())
        if val < best_val - 1e-18:
            best_val, best = val, cand
    return best, best_val


# ----------------------------------------------------------------------------
# learning the transform: regulariser, update rules, loops
# ----------------------------------------------------------------------------
def orth_penalty(T, lam):
    """lam * ||T T^T - I||_F / sqrt(d) for the block-diagonal T (d = nb*k, one norm over all
    blocks) and its gradient w.r.t. the blocks: with R = T T^T - I (symmetric),
    d||R||_F = <R, dR>/||R||_F and dR = dT T^T + T dT^T give 2 R T / ||R||_F.
    The gradient is taken as zero where the norm vanishes."""
    T = np.asarray(T, dtype=np.float64)
    nb, k, _ = T.shape
    R = T @ T.transpose(0, 2, 1) - np.eye(k)[None]
    n = float(np.sqrt((R * R).sum()))
    d = nb * k
    val = lam * n / np.sqrt(d)
    if n <= 1e-30:
        return val, np.zeros_like(T)
    return val, (lam / np.sqrt(d)) * 2.0 * (R @ T) / n


def sgd_step(T, g, lr):
    return T - lr * g


def adam_step(T, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One step of Adam (Kingma & Ba, Algorithm 1) with bias correction; t counts from 1."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return T - lr * mhat / (np.sqrt(vhat) + eps), m, v


def optimize_single(W, T0, bits, group, axis, rep, lr, steps, lam=0.0, normalize=True):
    """Gradient descent on the surrogate (plus the regulariser) for one matrix.  With
    ``normalize`` the surrogate is divided by ||W||_F^2 (it then bounds the squared RELATIVE
    l2 error), which makes the learning rate dimensionless.  Returns (T, history) where
    history[s] = (l2_sq, err_z_sq, w_sq, surrogate, penalty) evaluated at the T of step s."""
    W = np.asarray(W, dtype=np.float64)
    T = np.asarray(T0, dtype=np.float64).copy()
    hist = []
    for _ in range(steps):
        P = block_inverse(T)
        f = proxy_l2(W, T, P, bits, group, axis, rep)
        sur, g = surrogate(W, T, P, bits, group, axis, rep)
        pen, gp = orth_penalty(T, lam)
        if normalize:
            g = g / f["w_sq"]
        hist.append((f["l2_sq"], f["err_z_sq"], f["w_sq"], sur, pen))
        T = sgd_step(T, g + gp, lr)
    return T, np.array(hist)


def optimize_pair(A, B, T0, bits, group, rep, t, lr, steps, lam=0.0, beta1=0.1, beta2=0.999, eps=1e-8):
    """Adam on the LogSumExp surrogate (plus the regulariser) for a coupled pair.  Returns
    (T, history) with history[s] = (errU_sq, errV_sq, l2A_sq, l2B_sq, lse, penalty)."""
    T = np.asarray(T0, dtype=np.float64).copy()
    m = np.zeros_like(T)
    v = np.zeros_like(T)
    hist = []
    for s in range(steps):
        P = block_inverse(T)
        f = dual_lse(A, B, T, P, bits, group, rep, t)
        pen, gp = orth_penalty(T, lam)
        hist.append((f["errU_sq"], f["errV_sq"], f["l2A_sq"], f["l2B_sq"], f["lse"], pen))
        T, m, v = adam_step(T, f["gradT"] + gp, m, v, s + 1, lr, beta1, beta2, eps)
    return T, np.array(hist)


# ----------------------------------------------------------------------------
# randomized-Hadamard baseline
# ----------------------------------------------------------------------------
def hadamard_matrix(n):
    """Sylvester's construction: H_1 = [1], H_2m = [[H_m, H_m], [H_m, -H_m]] (n a power of two)."""
    H = np.ones((1, 1))
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    assert H.shape[0] == n
    return H


def hadamard_apply(W, signs, blk):
    """Z = W . blockdiag(D_b H / sqrt(blk)) along the columns: the elements of each block of `blk`
    consecutive columns are multiplied by their random signs, then by the normalised Hadamard
    matrix (an orthogonal transform)."""
    W = np.asarray(W, dtype=np.float64)
    R, C = W.shape
    H = hadamard_matrix(blk) / np.sqrt(blk)
    X = (W * np.asarray(signs, dtype=np.float64)[None, :]).reshape(R, C // blk, blk)
    return (X @ H).reshape(R, C)


def hadamard_baseline(W, signs, blk, bits, group, arith="f32"):
    """The 'random' row of the paper's block-size table: transform with randomized Hadamard blocks,
    quantize, transform back.  Returns dict(l2_sq, err_z_sq, w_sq, Z, Zhat); the transform is
    orthogonal, so the two errors coincide (the way back is written out here, not assumed)."""
    W = np.asarray(W, dtype=np.float64)
    Z = hadamard_apply(W, signs, blk)
    Zhat = quantize(Z, bits, group, COL, SYM, arith)
    E = Zhat - Z
    R, C = W.shape
    H = hadamard_matrix(blk) / np.sqrt(blk)
    D = ((E.reshape(R, C // blk, blk) @ H.T).reshape(R, C)) * np.asarray(signs, dtype=np.float64)[None, :]
    return dict(l2_sq=float((D * D).sum()), err_z_sq=float((E * E).sum()), w_sq=float((W * W).sum()),
                Z=Z, Zhat=Zhat)


# ----------------------------------------------------------------------------
# inference side of a single transformed matrix
# ----------------------------------------------------------------------------
def dequantize(codes, scales, group, axis=COL):
    """Symmetric grid: zhat = fl32(q * s), the scale of an element's group spread over the group."""
    q = np.asarray(codes).astype(np.float32)
    R, C = q.shape
    s = np.asarray(scales, dtype=np.float32)
    if axis == COL:
        g = C if group == 0 else group
        full = np.repeat(s.reshape(R, C // g), g, axis=1)
    else:
        g = R if group == 0 else group
        full = np.repeat(s.reshape(R // g, C), g, axis=0)
    return (q * full).astype(np.float64)


def infer_single(X, P, codes, scales, group):
    """Layer output with the quantized transformed weight (Sec. 4.1): Y^ = X M^-1 Q(MW).

    Orientation: the paper's weight is [in][out] and M acts on its left; here weights are [out][in] and
    Z = W . blockdiag(T) (axis COL), so Q(MW) = Zhat^T and M^-1 = blockdiag(P)^T with P = T^-1 blockwise.
    X: [n][in] activations; P: [nb][k][k] or None (no transform: the plain quantized layer);
    codes [out][in], scales [out][in/group].  Returns Y^ [n][out] (float64)."""
    X = np.asarray(X, dtype=np.float64)
    n, d = X.shape
    Zhat = dequantize(codes, scales, group, COL)            # [out][in]
    assert Zhat.shape[1] == d
    if P is None:
        XM = X
    else:
        P = np.asarray(P, dtype=np.float64)
        nb, k, _ = P.shape
        assert nb * k == d
        Minv = np.zeros((d, d))
        for b in range(nb):
            Minv[b * k:(b + 1) * k, b * k:(b + 1) * k] = P[b].T
        XM = X @ Minv
    return XM @ Zhat.T
