"""GPU parity: the inference side of a single transformed matrix (cafeq_infer_single) against the oracle.

Inputs (activations, inverse blocks, codes, scales) are the oracle's or synthetic; both sides read the
same float32 / int8 arrays.  Tolerance: the device forms x' = P x as a float32 dot product of k terms and
the output as a float32 sum over the inputs, so
  |y - y_ref| <= 2^-24 (k + 32) sum_c |zhat_c| (sum_j |P_cj| |x_j|)
(the standard bound of a two-level float32 dot product; 32 covers the 16-term chains, the tree over the
threads and the scale product)."""
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


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _bound(X, P, codes, scales, group, k):
    Za = np.abs(O.dequantize(codes, scales, group))
    Xa = np.abs(X.astype(np.float64))
    if P is None:
        xa = Xa
    else:
        nb = P.shape[0]
        xa = np.einsum("bij,tbj->tbi", np.abs(P.astype(np.float64)), Xa.reshape(len(X), nb, k)).reshape(len(X), -1)
    return (k + 32) * 2.0 ** -24 * (xa @ Za.T) + 1e-30


def _run(env, X, P, codes, scales, group):
    torch, cafeq = env
    Y = cafeq.infer_single(_dev(torch, X), None if P is None else _dev(torch, P), _dev(torch, codes),
                           _dev(torch, scales), group)
    torch.cuda.synchronize()
    return Y.cpu().numpy().astype(np.float64)


def _quantized(out, d, k, bits, group, seed):
    W = WL.student_t3((out, d), seed)
    T = WL.perturbed_blocks(d // k, k, seed + 1, eps=0.1)
    P = O.block_inverse(T).astype(np.float32)
    Z = O.blockdiag_apply(W, T, O.COL)
    codes, scales, _ = O.rtn_sym(Z, bits, group, O.COL)
    return P, codes, scales.astype(np.float32)


def _check(env, X, P, codes, scales, group, k):
    Y = _run(env, X, P, codes, scales, group)
    ref = O.infer_single(X, P, codes, scales, group)
    err = np.abs(Y - ref)
    bound = _bound(X, P, codes, scales, group, k)
    assert np.all(err <= bound), "max err/bound %.3g" % (err / bound).max()
    print("max |err| / bound = %.3f, max rel to |y|max = %.2e" % ((err / bound).max(), err.max() / np.abs(ref).max()))
    return Y


@pytest.mark.parametrize("k", [32, 64, 128, 256])
@pytest.mark.parametrize("n", [1, 2, 3, 5])
def test_block_sizes_and_token_counts(env, k, n):
    out, d, group = 37, 4 * 256 + (k if k < 256 else 256), 32
    P, codes, scales = _quantized(out, d, k, 4, group, 100 + k + n)
    X = WL.gaussian((n, d), 7 + n, std=1.0)
    _check(env, X, P, codes, scales, group, k)


@pytest.mark.parametrize("d,group", [(1088, 16), (1088, 0), (3072, 128), (4096 + 512, 256), (9216, 64)])
def test_input_widths_cover_the_thread_shapes_and_ragged_chunks(env, d, group):
    k = 64
    P, codes, scales = _quantized(21, d, k, 3, group, d + group)
    for n in (1, 4):
        X = WL.gaussian((n, d), 17 + n, std=1.0)
        _check(env, X, P, codes, scales, group, k)


def test_many_tokens_and_strided_activations(env):
    torch, cafeq = env
    k, d, out, group = 128, 1024, 70, 128
    P, codes, scales = _quantized(out, d, k, 4, group, 900)
    n = 19
    Xfull = WL.gaussian((n, d + 8), 901, std=1.0)
    Xd = _dev(torch, Xfull)[:, :d]                      # leading dimension d + 8
    Y = cafeq.infer_single(Xd, _dev(torch, P), _dev(torch, codes), _dev(torch, scales), group)
    torch.cuda.synchronize()
    X = np.ascontiguousarray(Xfull[:, :d])
    ref = O.infer_single(X, P, codes, scales, group)
    assert np.all(np.abs(Y.cpu().numpy() - ref) <= _bound(X, P, codes, scales, group, k))


def test_without_a_transform_it_is_the_plain_quantized_layer(env):
    d, out, group = 2048, 50, 64
    W = WL.student_t3((out, d), 31)
    codes, scales, Zhat = O.rtn_sym(W, 4, group, O.COL)
    scales = scales.astype(np.float32)
    X = WL.gaussian((2, d), 32, std=1.0)
    Y = _check(env, X, None, codes, scales, group, 0)
    np.testing.assert_allclose(Y, X.astype(np.float64) @ Zhat.T, rtol=0, atol=1e-4 * np.abs(Y).max())


def test_a_weight_on_the_grid_is_reproduced(env):
    # integer codes, power-of-two scales, signed-permutation blocks, integer activations: every product
    # and partial sum is an exact float32 number, so the device must return X W^T exactly
    rng = np.random.default_rng(5)
    nb, k, out, group = 8, 32, 9, 32
    T = np.zeros((nb, k, k))
    for b in range(nb):
        T[b][np.arange(k), rng.permutation(k)] = rng.choice([-1.0, 1.0], k) * 2.0 ** rng.integers(-1, 2)
    P = O.block_inverse(T).astype(np.float32)
    codes = rng.integers(-7, 8, (out, nb * k)).astype(np.int8)
    scales = (2.0 ** rng.integers(-4, 0, (out, nb * k // group))).astype(np.float32)
    W = O.blockdiag_apply(O.dequantize(codes, scales, group), P, O.COL)
    X = rng.integers(-3, 4, (3, nb * k)).astype(np.float32)
    Y = _run(env, X, P, codes, scales, group)
    np.testing.assert_array_equal(Y, X.astype(np.float64) @ W.T)


def test_repeated_calls_are_bit_identical(env):
    torch, cafeq = env
    P, codes, scales = _quantized(64, 2048, 128, 4, 128, 77)
    X = WL.gaussian((4, 2048), 78, std=1.0)
    a = _run(env, X, P, codes, scales, 128)
    b = _run(env, X, P, codes, scales, 128)
    np.testing.assert_array_equal(a, b)


def test_down_projection_of_the_2b_shaped_model_at_full_size(env):
    # the matrix of the paper's block-size table: input dimension 9216, output dimension 2304
    rows, cols, k, group, bits = 2304, 9216, 128, 128, 4
    W = WL.config2(rows, cols)["W"]
    T = WL.perturbed_blocks(cols // k, k, 41, eps=0.1)
    P = O.block_inverse(T).astype(np.float32)
    codes, scales, _ = O.rtn_sym(O.blockdiag_apply(W, T, O.COL), bits, group, O.COL)
    scales = scales.astype(np.float32)
    for n in (1, 4):
        X = WL.gaussian((n, cols), 42 + n, std=1.0)
        _check(env, X, P, codes, scales, group, k)


def test_square_14336_matrix_with_synthetic_codes(env):
    # full-size property check at the largest single-matrix shape of the workloads: random 3-bit codes
    # and log-normal scales stand in for a quantized weight (the entry point sees only codes and scales)
    rng = np.random.default_rng(11)
    d, k, group = 14336, 128, 128
    codes = rng.integers(-4, 4, (d, d), dtype=np.int8)
    scales = np.exp(rng.normal(-5.0, 0.5, (d, d // group))).astype(np.float32)
    P = O.block_inverse(WL.perturbed_blocks(d // k, k, 12, eps=0.1)).astype(np.float32)
    X = WL.gaussian((1, d), 13, std=1.0)
    _check(env, X, P, codes, scales, group, k)
