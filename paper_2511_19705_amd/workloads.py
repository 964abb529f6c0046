"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

This module only *generates data*: weight matrices with the shapes and outlier
structure of Gemma-2 layers (stand-ins for the real weights the paper's
experiments section uses, which are not available offline) and random-rotation
initial transforms (the paper's section on single-matrix transforms initialises
every diagonal block to a random rotation).  It holds none of the method's
arithmetic: no quantizer, no transform application, no loss.  Everything is
NumPy on the host; callers upload the arrays they need.

Layout convention (used by the whole repository): a weight is a row-major 2-D
array ``W[R][C]``; a transform is ``nb`` dense ``k x k`` blocks ``T[nb][k][k]``
acting along one axis of ``W``:

* axis ``COL`` (0): the contiguous axis, ``Z = W . blockdiag(T)``, ``nb*k == C``;
* axis ``ROW`` (1): the strided axis, ``Z = blockdiag(T) . W``, ``nb*k*rep == R``
  (``rep`` consecutive row-blocks share one transform block: grouped-query heads).
"""
from __future__ import annotations

import numpy as np

AXIS_COL = 0
AXIS_ROW = 1


# ----------------------------------------------------------------------------
# elementary generators
# ----------------------------------------------------------------------------
def gaussian(shape, seed, std=0.02):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(np.float32)


def student_t3(shape, seed, std=0.02):
    """Student-t, 3 degrees of freedom, scaled so the *population* std is ``std``
    (variance of t_3 is 3)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_t(3, size=shape) * (std / np.sqrt(3.0))).astype(np.float32)


def scale_random_entries(W, frac, factor, seed):
    """Multiply a fraction ``frac`` of the entries (chosen uniformly without
    replacement) by ``factor`` in place; returns the flat indices."""
    rng = np.random.default_rng(seed)
    n = W.size
    cnt = max(1, int(round(frac * n)))
    idx = rng.choice(n, size=cnt, replace=False)
    flat = W.reshape(-1)
    flat[idx] *= np.float32(factor)
    return idx


def scale_random_columns(W, count, factor, seed):
    rng = np.random.default_rng(seed)
    cols = rng.choice(W.shape[1], size=count, replace=False)
    W[:, cols] *= np.float32(factor)
    return cols


def haar_blocks(nb, k, seed):
    """``nb`` independent Haar-distributed orthogonal ``k x k`` blocks:
    QR of a Gaussian matrix with the sign of diag(R) fixed positive."""
    rng = np.random.default_rng(seed)
    out = np.empty((nb, k, k), dtype=np.float64)
    for b in range(nb):
        g = rng.standard_normal((k, k))
        q, r = np.linalg.qr(g)
        q = q * np.sign(np.diag(r))[None, :]
        out[b] = q
    return out.astype(np.float32)


def perturbed_blocks(nb, k, seed, eps=0.05):
    """Rotation blocks pushed off the orthogonal manifold (a transform part-way
    through learning): ``Q (I + eps*G/sqrt(k))``.  Well conditioned for small eps."""
    rng = np.random.default_rng(seed + 7919)
    q = haar_blocks(nb, k, seed).astype(np.float64)
    g = rng.standard_normal((nb, k, k)) * (eps / np.sqrt(k))
    return (q @ (np.eye(k)[None] + g)).astype(np.float32)


def to_bf16_bits(x):
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# the five workloads (full size) and scaled-down twins for element-wise parity
# ----------------------------------------------------------------------------
def config1():
    """256x256 Gaussian, 0.1% entries x20; 8 rotation blocks of 32; 4 bit, group 32."""
    W = gaussian((256, 256), 101)
    scale_random_entries(W, 0.001, 20.0, 1101)
    return dict(name="c1_256x256_k32_g32_b4", W=W, T=haar_blocks(8, 32, 102),
                k=32, group=32, bits=(4,), axis=AXIS_COL)


def config2(rows=2304, cols=9216):
    """Gemma-2-2B-shaped down projection: Student-t(3), 8 outlier input columns x10;
    rotation blocks of 64; 4 and 3 bit, group 128."""
    W = student_t3((rows, cols), 201)
    scale_random_columns(W, 8, 10.0, 1201)
    return dict(name="c2_%dx%d_k64_g128" % (rows, cols), W=W,
                T=haar_blocks(cols // 64, 64, 202), k=64, group=128,
                bits=(4, 3), axis=AXIS_COL)


def config3(d_model=3584, d_ff=14336, k=128):
    """Gemma-2-9B-shaped MLP pair sharing one block-diagonal transform on the
    intermediate dimension: A = down [d_model x d_ff] gets T on its columns,
    B = up [d_ff x d_model] gets T^-1 on its rows.  3 bit, group 128."""
    A = student_t3((d_model, d_ff), 301)
    scale_random_entries(A, 0.0005, 20.0, 1301)
    B = student_t3((d_ff, d_model), 302)
    scale_random_entries(B, 0.0005, 20.0, 1302)
    return dict(name="c3_pair_%dx%d_k%d_g128_b3" % (d_model, d_ff, k), A=A, B=B,
                T=haar_blocks(d_ff // k, k, 303), k=k, rep=1, group=128, bits=(3,))


def config4(d_model=3584, n_kv=8, n_q=16, head=256):
    """Gemma-2-9B-shaped attention V/O pair: V [d_model x n_kv*head] (columns
    transformed), O [n_q*head x d_model] (rows transformed, `rep = n_q/n_kv`
    query heads share a kv head's block).  Gaussian with 2 outlier head-dim
    channels per kv head (x8), the same channel in V's columns and O's rows.
    4 bit, group 64, adaptive rounding."""
    rep = n_q // n_kv
    A = gaussian((d_model, n_kv * head), 401)
    B = gaussian((n_q * head, d_model), 402)
    rng = np.random.default_rng(1401)
    for h in range(n_kv):
        ch = rng.choice(head, size=2, replace=False)
        for c in ch:
            A[:, h * head + c] *= np.float32(8.0)
            for q in range(rep):
                B[(h * rep + q) * head + c, :] *= np.float32(8.0)
    return dict(name="c4_vo_%d_kv%d_q%d_h%d_g64_b4" % (d_model, n_kv, n_q, head),
                A=A, B=B, T=haar_blocks(n_kv, head, 403), k=head, rep=rep,
                group=64, bits=(4,))


def config5_shapes(d_model=4608, d_ff=36864, n_q=32, n_kv=16, head=128):
    """Gemma-2-27B-shaped decoder layer: (name, rows, cols, axis, role)."""
    return [
        ("q", n_q * head, d_model, AXIS_COL, "single"),
        ("k", n_kv * head, d_model, AXIS_COL, "single"),
        ("gate", d_ff, d_model, AXIS_COL, "single"),
        ("down", d_model, d_ff, AXIS_COL, "pairA_mlp"),
        ("up", d_ff, d_model, AXIS_ROW, "pairB_mlp"),
        ("v", d_model, n_kv * head, AXIS_COL, "pairA_vo"),
        ("o", n_q * head, d_model, AXIS_ROW, "pairB_vo"),
    ]


def config5_meta(scale=1):
    """Sizes and transforms of the 27B-shaped layer (``scale`` divides d_model and d_ff)."""
    d_model, d_ff = 4608 // scale, 36864 // scale
    n_q, n_kv, head = 32 // scale if scale <= 2 else max(2, 32 // scale), \
        16 // scale if scale <= 2 else max(1, 16 // scale), 128
    return dict(k=128, group=128, bits=(3, 4), d_model=d_model, d_ff=d_ff,
                n_q=n_q, n_kv=n_kv, head=head, rep=n_q // n_kv)


def config5_transform(which, scale=1):
    """Haar blocks of the layer: 'single' (input dim of q, k, gate), 'mlp' (down/up pair),
    'vo' (one block per kv head)."""
    m = config5_meta(scale)
    if which == "single":
        return haar_blocks(m["d_model"] // 128, 128, 508)
    if which == "mlp":
        return haar_blocks(m["d_ff"] // 128, 128, 509)
    return haar_blocks(m["n_kv"], 128, 510)


def config5_tensor(name, scale=1):
    """One weight of the 27B-shaped layer as bf16 bit patterns (uint16) + its axis and role."""
    m = config5_meta(scale)
    for i, (nm, r, c, axis, role) in enumerate(
            config5_shapes(m["d_model"], m["d_ff"], m["n_q"], m["n_kv"], m["head"])):
        if nm == name:
            return dict(bits16=to_bf16_bits(student_t3((r, c), 501 + i)), axis=axis, role=role)
    raise KeyError(name)


def config5(scale=1):
    """All seven weights of the 27B-shaped layer as bf16 bit patterns (uint16).
    ``scale`` divides d_model and d_ff (for CPU-sized twins)."""
    m = config5_meta(scale)
    out = {}
    for nm, _, _, _, _ in config5_shapes(m["d_model"], m["d_ff"], m["n_q"], m["n_kv"], m["head"]):
        out[nm] = config5_tensor(nm, scale)
    out["_meta"] = dict(m, T_single=config5_transform("single", scale),
                        T_mlp=config5_transform("mlp", scale), T_vo=config5_transform("vo", scale))
    return out


def small_single(rows, cols, k, seed, heavy=True, eps=0.0):
    """A CPU-sized single-matrix case with the same value recipe as config 2."""
    W = student_t3((rows, cols), seed) if heavy else gaussian((rows, cols), seed)
    scale_random_columns(W, max(1, cols // 1024), 10.0, seed + 1000)
    T = perturbed_blocks(cols // k, k, seed + 1, eps) if eps else haar_blocks(cols // k, k, seed + 1)
    return W, T


def small_pair(d_model, d_mid, k, rep, seed, eps=0.0):
    """A CPU-sized pair: A [d_model x d_mid] (COL), B [d_mid*rep x d_model] (ROW)."""
    A = student_t3((d_model, d_mid), seed)
    B = student_t3((d_mid * rep, d_model), seed + 1)
    scale_random_entries(A, 0.0005, 20.0, seed + 1000)
    scale_random_entries(B, 0.0005, 20.0, seed + 1001)
    nb = d_mid // k
    T = perturbed_blocks(nb, k, seed + 2, eps) if eps else haar_blocks(nb, k, seed + 2)
    return A, B, T


def random_signs(n, seed):
    """n random +-1 values (float32): the diagonal of a randomized Hadamard transform."""
    rng = np.random.default_rng(seed)
    return (rng.integers(0, 2, size=n).astype(np.float32) * 2.0 - 1.0)
