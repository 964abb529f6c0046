"""Pins for the oracle's quantizers: Eq. (1), Eq. (2), the symmetric grid's
invariants, brute force over all levels, and the group layouts."""
import os

import numpy as np
import pytest

from oracle import cafeq_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed, heavy=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, size=shape) if heavy else rng.standard_normal(shape)
    return (x * 0.02).astype(np.float32)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("axis,group", [(O.COL, 32), (O.COL, 0), (O.ROW, 16), (O.ROW, 0)])
def test_sym_invariants(bits, axis, group):
    Z = _rand((64, 96), 1 + bits)
    qmax, qmin = 2 ** (bits - 1) - 1, -(2 ** (bits - 1))
    for arith in ("f64", "f32"):
        codes, scales, zhat = O.rtn_sym(Z, bits, group, axis, arith)
        assert codes.dtype == np.int8 and codes.min() >= qmin and codes.max() <= qmax
        # per-element error <= s/2 (tiny slack for the single-precision recipe)
        g = group if group else (Z.shape[1] if axis == O.COL else Z.shape[0])
        s_elem = np.repeat(scales, g, axis=1 if axis == O.COL else 0)
        slack = 0.0 if arith == "f64" else 4 * 2.0 ** -24 * qmax
        err = np.abs(zhat - Z.astype(np.float64))
        assert np.all(err <= 0.5 * s_elem * (1 + slack) + 1e-300)
        # the element carrying the absmax maps to +-qmax exactly and is reproduced
        Zg = O._to_groups(Z.astype(np.float64), axis, group)
        cg = O._to_groups(codes.astype(np.float64), axis, group)
        idx = np.argmax(np.abs(Zg), axis=1)
        r = np.arange(Zg.shape[0])
        assert np.all(np.abs(cg[r, idx]) == qmax)
        zg = O._to_groups(zhat, axis, group)
        np.testing.assert_allclose(zg[r, idx], Zg[r, idx], rtol=3e-7)


def test_sym_matches_bruteforce_nearest_level():
    # enumerate every representable level and take the nearest: the definition of RTN
    rng = np.random.default_rng(5)
    for bits in (2, 3, 4):
        Z = rng.standard_normal((6, 8))
        codes, scales, zhat = O.rtn_sym(Z, bits, 4, O.COL, "f64")
        qmax, qmin = 2 ** (bits - 1) - 1, -(2 ** (bits - 1))
        for r in range(6):
            for c in range(8):
                s = scales[r, c // 4]
                levels = np.arange(qmin, qmax + 1) * s
                best = levels[np.argmin(np.abs(levels - Z[r, c]))]
                assert abs(best - zhat[r, c]) < 1e-15


def test_sym_zero_group_and_ties_to_even():
    Z = np.zeros((2, 8))
    Z[1] = [7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]      # absmax 7, qmax 7 -> s = 1
    codes, scales, zhat = O.rtn_sym(Z, 4, 8, O.COL, "f32")
    assert np.all(codes[0] == 0) and scales[0, 0] == 0 and np.all(zhat[0] == 0)
    assert list(codes[1]) == [7, 0, 2, 2, 0, -2, -2, 4]


def test_f32_recipe_differs_from_exact_only_at_ties():
    Z = _rand((256, 512), 11)
    c64, _, _ = O.rtn_sym(Z, 4, 128, O.COL, "f64")
    c32, s32, _ = O.rtn_sym(Z, 4, 128, O.COL, "f32")
    diff = c64 != c32
    assert diff.mean() <= 1e-5
    if diff.any():
        assert np.abs(c64.astype(int) - c32.astype(int))[diff].max() == 1
        s_el = np.repeat(s32.astype(np.float64), 128, axis=1)
        frac = np.abs(Z.astype(np.float64)[diff] / s_el[diff])
        assert np.all(np.abs(frac - np.floor(frac) - 0.5) < 1e-5)


def test_row_axis_layout_against_loops():
    Z = _rand((32, 5), 3).astype(np.float64)
    g, bits = 8, 3
    codes, scales, zhat = O.rtn_sym(Z, bits, g, O.ROW, "f64")
    assert scales.shape == (4, 5)
    qmax = 3
    for c in range(5):
        for gi in range(4):
            col = Z[gi * g:(gi + 1) * g, c]
            a = np.max(np.abs(col))
            assert abs(scales[gi, c] - a / qmax) < 1e-18
            for r in range(g):
                q = int(np.clip(np.rint(col[r] / (a / qmax)), -4, 3))
                assert codes[gi * g + r, c] == q
                assert abs(zhat[gi * g + r, c] - q * a / qmax) < 1e-15


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_asym_error_bound_eq2(bits):
    Z = _rand((40, 64), 21 + bits).astype(np.float64)
    for axis, group in ((O.COL, 16), (O.ROW, 8), (O.COL, 0), (O.COL, -1)):
        codes, s, lo, zhat = O.rtn_asym(Z, bits, group, axis)
        Zg = O._to_groups(Z, axis, group)
        zg = O._to_groups(zhat, axis, group)
        rng_ = Zg.max(axis=1) - Zg.min(axis=1)
        bound1 = rng_ / (2 * (2 ** bits - 1))
        bound2 = np.max(np.abs(Zg), axis=1) / (2 ** bits - 1)
        err = np.abs(zg - Zg).max(axis=1)
        assert np.all(err <= bound1 * (1 + 1e-12))
        assert np.all(bound1 <= bound2 * (1 + 1e-12))
        assert codes.min() >= 0 and codes.max() <= 2 ** bits - 1


def test_asym_f32_recipe_differs_from_exact_only_at_ties():
    Z = _rand((256, 512), 13)
    c64, s64, lo64, z64 = O.rtn_asym(Z, 4, 128, O.COL, "f64")
    c32, s32, lo32, z32 = O.rtn_asym(Z, 4, 128, O.COL, "f32")
    np.testing.assert_array_equal(lo32, lo64)                      # min / max are exact in float32
    np.testing.assert_allclose(s32, s64, rtol=2e-7)
    diff = c64 != c32
    assert diff.mean() <= 1e-4
    if diff.any():
        assert np.abs(c64.astype(int) - c32.astype(int))[diff].max() == 1
        s_el = np.repeat(s64, 128, axis=1)
        l_el = np.repeat(lo64, 128, axis=1)
        frac = (Z.astype(np.float64)[diff] - l_el[diff]) / s_el[diff]
        assert np.all(np.abs(frac - np.floor(frac) - 0.5) < 1e-4)
    # the dequantized value obeys Eq. (2)'s bound up to float32 rounding
    rng_ = np.repeat(15.0 * s64, 128, axis=1)
    assert np.all(np.abs(z32 - Z) <= rng_ / 30.0 * (1 + 1e-5) + 1e-9)
    # a constant group: code 0, value reproduced exactly
    C = np.full((4, 128), 0.37, dtype=np.float32)
    c, s_, lo_, zq = O.rtn_asym(C, 3, 128, O.COL, "f32")
    assert c.max() == 0 and float(s_.max()) == 0.0
    np.testing.assert_array_equal(zq, C.astype(np.float64))


def _read_gold(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def test_toy_example_independent_rounding():
    g = _read_gold("toy_example.txt")
    W = np.diag([g["w_diag0"], g["w_diag1"]])
    codes, s, lo, what = O.rtn_asym(W, int(g["bits"]), -1, O.COL)
    np.testing.assert_array_equal(what, np.eye(2))
    p, _ = O.pqe(W, W, what, what, k=2)
    assert abs(p - g["pqe_independent"]) < 1e-12


def test_denormal_absmax_group_stays_finite():
    # the single-precision recipe caps inv = fl(qmax / a) at FLT_MAX: for a denormal absmax the uncapped
    # quotient is inf and 0 * inf would be NaN.  With the cap every product is finite, so every code is a
    # finite integer in range and the dequantized values are finite; a normal group next to it is untouched.
    tiny = np.float32(1e-42)
    Z = np.array([[tiny, 0.0, -tiny, 0.0, 1.0, -0.5, 0.25, 0.0]], dtype=np.float32)
    codes, scales, zh = O.rtn_sym(Z, 4, 4, O.COL, "f32")
    assert np.all(np.isfinite(zh)) and np.all(np.isfinite(scales))
    assert codes.min() >= -8 and codes.max() <= 7
    np.testing.assert_array_equal(codes[0, 4:], [7, -4, 2, 0])      # 1 -> qmax, -0.5*7 = -3.5 -> -4 (even), 0.25*7 = 1.75 -> 2
    assert np.all(np.abs(zh[0, :4] - Z[0, :4].astype(np.float64)) <= float(tiny))
