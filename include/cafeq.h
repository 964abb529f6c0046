/*
 * cafeq.h -- C ABI of the MI355X (gfx950) CafeQ hot-path library.
 *
 * CafeQ (arxiv 2511.19705) learns a block-diagonal transform M per weight matrix so
 * that round-to-nearest quantization of the transformed weight loses less, using
 * losses that need no calibration data.  This library evaluates the inner loop of
 * that optimisation on one GPU:
 *   transform -> per-group absmax scale -> b-bit round-to-nearest -> dequantize ->
 *   inverse transform -> reduce the data-free proxy losses and the gradient of the
 *   differentiable surrogate with respect to the transform,
 * for a single matrix (paper Sec. 4.1), for a coupled pair sharing M / M^-1
 * (Sec. 4.2), and one iteration of the alternating adaptive rounding (Sec. 5, Alg. 1).
 *
 * Conventions (all entry points)
 *  - Weights are row-major 2-D arrays W[rows][cols] with leading dimension `ld`
 *    (elements), float32 or bfloat16 storage; all arithmetic is float32 (float64 for
 *    final reductions and for the small k x k solves).
 *  - A transform is `nb` dense k x k float32 blocks, T[nb][k][k] row-major, with its
 *    blockwise inverse Tinv[nb][k][k].  It acts along one axis of W:
 *      CAFEQ_AXIS_COL: Z = W . blockdiag(X)      (nb*k == cols; contiguous axis)
 *      CAFEQ_AXIS_ROW: Z = blockdiag(X) . W      (nb*rep*k == rows; row-block q of k
 *                      rows uses block q / rep -- grouped-query heads share a block)
 *    With PyTorch's [out][in] weight layout the paper's M (acting on the contraction
 *    dimension) is T^T on AXIS_COL.
 *  - Quantization groups are `group` consecutive elements along cfg->axis
 *    (group == 0: the whole line).  Scale layout: AXIS_COL -> scales[rows][cols/group],
 *    AXIS_ROW -> scales[rows/group][cols].  Codes are one int8 per element, [rows][cols]
 *    dense (leading dimension == cols).
 *  - Symmetric grid (CAFEQ_Q_SYM_ABSMAX): a = max|z| over the group, qmax = 2^(b-1)-1,
 *    inv = fl32(qmax / a), q = clamp(rint(fl32(z*inv)), -2^(b-1), qmax) (ties to even),
 *    s = fl32(a / qmax), dequantized value fl32(q*s); a == 0 gives s = 0, q = 0.
 *  - Every pointer named in a signature is a DEVICE pointer owned by the caller unless
 *    stated otherwise; descriptor structs themselves are host memory, read during the
 *    call only.  Nothing is allocated or freed by the library (no device memory, no events,
 *    no streams); scratch memory is the caller's `ws` buffer, sized by
 *    cafeq_workspace_bytes() and 256-byte aligned.
 *  - `stream` is a hipStream_t (NULL = default stream).  Calls enqueue work and return;
 *    outputs are valid once the stream has been synchronised.  Results (losses too) are
 *    written to device memory, never returned through the host.
 *  - Return value: CAFEQ_OK (0) or a negative cafeq_status.  Argument errors are
 *    detected on the host before anything is launched.  No exceptions cross the ABI.
 *  - Calls that share a `ws` buffer must be ordered on one stream.
 */
#ifndef CAFEQ_H
#define CAFEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CAFEQ_OK = 0,
  CAFEQ_ERR_INVALID_ARG = -1, /* NULL where a pointer is required, bad enum value   */
  CAFEQ_ERR_BAD_SHAPE = -2,   /* sizes not divisible as the operation requires      */
  CAFEQ_ERR_BAD_ALIGN = -3,   /* pointer / leading dimension alignment              */
  CAFEQ_ERR_UNSUPPORTED = -4, /* valid request this build has no kernel for         */
  CAFEQ_ERR_SINGULAR = -5,    /* reserved for host-visible singularity reports      */
  CAFEQ_ERR_LAUNCH = -6,      /* the HIP runtime refused a launch                   */
  CAFEQ_ERR_WORKSPACE = -7    /* ws is NULL or smaller than cafeq_workspace_bytes() */
} cafeq_status;

typedef enum { CAFEQ_F32 = 0, CAFEQ_BF16 = 1 } cafeq_dtype;
typedef enum { CAFEQ_AXIS_COL = 0, CAFEQ_AXIS_ROW = 1 } cafeq_axis;
typedef enum { CAFEQ_SIDE_T = 0, CAFEQ_SIDE_TINV = 1 } cafeq_side;
typedef enum { CAFEQ_Q_SYM_ABSMAX = 0, CAFEQ_Q_ASYM_MINMAX = 1 } cafeq_qmode;

/* Row-major matrix view. data: device pointer, 16-byte aligned; ld in elements, a
 * multiple of 4 (float32) or 8 (bfloat16); dtype: cafeq_dtype.
 * prepared: NULL, or a device buffer written by cafeq_prepare_weights() for this matrix (same data,
 * shape and the axis the call transforms).  The weights are constant over the thousands of loss
 * evaluations of a learning run (paper Sec. 4.1, Sec. 4.2); with a prepared copy the loss pass of
 * cafeq_proxy_loss_fwd_bwd / cafeq_dual_proxy_loss_fwd_bwd / cafeq_optimize_* reads them in the form
 * the matrix cores consume (where a kernel for it exists: blocks of 128, groups up to 128, up to
 * 4 bits; ignored otherwise).  `data` must stay valid either way: the gradient pass and every other
 * configuration read it.  Entry points that do not mention it ignore the field. */
typedef struct {
  const void* data;
  int64_t rows, cols, ld;
  int32_t dtype;
  const void* prepared;
} cafeq_mat;

/* Block-diagonal transform. T and Tinv: device, [nb][k][k] float32, 16-byte aligned.
 * k in {32, 64, 128, 256}, or one of the smaller sizes of the paper's block-size sweep, {2, 4, 8, 16}: those
 * are taken by cafeq_block_inverse, cafeq_apply_transform, cafeq_proxy_loss_fwd_bwd,
 * cafeq_dual_proxy_loss_fwd_bwd (rep = 1), cafeq_orth_penalty and the cafeq_optimize_* loops, which run every
 * 32 / k consecutive blocks as one block-diagonal block of 32 (the axis a multiple of 32; for
 * cafeq_block_inverse and cafeq_orth_penalty nb a multiple of 32 / k; status of cafeq_block_inverse is then
 * per run of 32 / k blocks); Alg. 1 and the paired error need k >= 32.
 * rep >= 1: number of consecutive row-blocks sharing one block (AXIS_ROW only; must be 1 on AXIS_COL). */
typedef struct {
  const float* T;
  const float* Tinv;
  int32_t k, nb, rep;
} cafeq_xform;

/* bits in [2, 8]; group: elements per scale along `axis` (0 = whole line);
 * axis: cafeq_axis; mode: cafeq_qmode.  CAFEQ_Q_ASYM_MINMAX, the min/max grid of the paper's Eq. (1), is
 * taken by cafeq_proxy_loss_fwd_bwd, cafeq_dual_proxy_loss_fwd_bwd and the two cafeq_optimize_* loops (see
 * there for the output layout); the untransformed quantizer on that grid is cafeq_rtn_quantize_minmax; the
 * other calls return CAFEQ_ERR_UNSUPPORTED for it. */
typedef struct {
  int32_t bits, group, axis, mode;
} cafeq_quant_cfg;

typedef enum {
  CAFEQ_CALL_RTN_QUANTIZE = 0,
  CAFEQ_CALL_PROXY_LOSS = 1,
  CAFEQ_CALL_DUAL_PROXY_LOSS = 2,
  CAFEQ_CALL_ADAPTIVE_ROUND = 3,
  CAFEQ_CALL_BLOCK_INVERSE = 4,  /* reads x->k and x->nb only */
  CAFEQ_CALL_APPLY_TRANSFORM = 5, /* reads x->k and x->nb only */
  CAFEQ_CALL_ORTH_PENALTY = 6,    /* reads x->k and x->nb only */
  CAFEQ_CALL_OPTIMIZE_SINGLE = 7, /* as CAFEQ_CALL_PROXY_LOSS */
  CAFEQ_CALL_OPTIMIZE_PAIR = 8,   /* as CAFEQ_CALL_DUAL_PROXY_LOSS */
  CAFEQ_CALL_PQE = 9              /* as CAFEQ_CALL_ADAPTIVE_ROUND */
} cafeq_call_id;

const char* cafeq_strerror(int status);
/* Library version as major*10000 + minor*100 + patch. */
int cafeq_version(void);

/* Bytes of scratch the given call needs for these arguments (0 on invalid input).
 * `a` is the only matrix for single-matrix calls; `b` and `x` may be NULL where the
 * call does not use them.  Only shapes are read, data pointers are ignored. */
size_t cafeq_workspace_bytes(int call_id, const cafeq_mat* a, const cafeq_mat* b,
                             const cafeq_xform* x, const cafeq_quant_cfg* cfg);

/* Blockwise inverse and the squared norms the surrogate needs (paper Sec. 4.1: the
 * (M^-1)_{ij}^2 factors).  Tinv[nb][k][k] = T^-1 per block (Gauss-Jordan with partial
 * pivoting, float64 internally; a block verified to be a rotation to float32 accuracy --
 * max |I - T T^T| <= 2e-6 -- is inverted by transposition; blocks of 256 are eliminated in float32 with one
 * Newton step on float64 residuals, and those near a scaled rotation are first tried with Newton-Schulz rounds from
 * T^T ||T||_F^-2 k, kept only where ||I - T X||_F <= 3e-4 afterwards).  rho_row[nb*k] / rho_col[nb*k] (either may be NULL):
 * squared row / column norms of Tinv.  status[nb] (may be NULL): 0 ok, 1 singular to
 * working precision (Tinv, rho_row and rho_col of that block are then zero).
 * k as in cafeq_xform (else CAFEQ_ERR_UNSUPPORTED). */
int cafeq_block_inverse(const float* T, int k, int nb, float* Tinv, float* rho_row,
                        float* rho_col, int* status, void* ws, void* stream);

/* Plain per-group round-to-nearest of W (paper Eq. (1)'s rounding rule on the symmetric
 * grid above; no transform).  codes[rows][cols], scales (layout above); err_sq[1]
 * (may be NULL) receives sum (dequant - w)^2.  Any group size dividing the line. */
int cafeq_rtn_quantize(const cafeq_mat* W, const cafeq_quant_cfg* cfg, int8_t* codes,
                       float* scales, float* err_sq, void* ws, void* stream);

/* cafeq_rtn_quantize for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same inputs, outputs
 * and arithmetic as cafeq_rtn_quantize; the float64 squared-error partials (one per workgroup) go to a
 * device array built into the library (512 KB per GPU, held until the process ends) instead of `ws`.
 * The call allocates and frees nothing.  With err_sq != NULL the matrix may hold at most
 * 65536 * 1024 * 4 elements along the contiguous axis' fast kernel and 65536 tiles of 16 rows x 256
 * columns (precisely: at most 65536 partials; larger inputs return CAFEQ_ERR_WORKSPACE before anything
 * is launched); with err_sq == NULL there is no limit.  Every call on a GPU shares that GPU's array:
 * calls that overlap on one GPU (different streams, different threads) race on it and must be
 * ordered by the caller.  Nothing needs clearing between calls (every partial is rewritten). */
int cafeq_rtn_quantize_static(const cafeq_mat* W, const cafeq_quant_cfg* cfg, int8_t* codes,
                              float* scales, float* err_sq, void* stream);

/* The uniform min/max quantizer exactly as the paper's Eq. (1) states it, per group:
 *   s = (max - min) / (2^b - 1),  q = nearest_int((w - min) / s) in [0, 2^b - 1],  w^ = s q + min.
 * Single-precision recipe: r = fl(max - min), inv = min(fl((2^b-1) / r), FLT_MAX) (0 for a constant
 * group, whose codes are 0), q = clamp(rint(fl(fl(w - min) * inv))), s = fl(r / (2^b-1)),
 * w^ = fl(fl(q s) + min); ties to even.  codes: unsigned bytes [rows][cols]; scales and mins
 * (either may be NULL) in the layout of cafeq_rtn_quantize's scales; err_sq as there.
 * bits in [1, 8]; cfg->mode is ignored; any group length dividing the line, 0 = the whole line
 * (the per-channel setting of the paper's experiments). */
int cafeq_rtn_quantize_minmax(const cafeq_mat* W, const cafeq_quant_cfg* cfg, uint8_t* codes,
                              float* scales, float* mins, float* err_sq, void* ws, void* stream);

/* The paper's "random" comparison (caption of the block-size table in Sec. 4.1: a block-diagonal
 * transform with blocks of 1024 whose blocks are randomized Hadamard matrices): every block of
 * `block` (256, 512 or 1024) consecutive columns of W is multiplied by its random signs
 * (signs[cols], +-1) and by the normalised Walsh-Hadamard matrix in Sylvester's ordering, then
 * quantized as in cafeq_rtn_quantize (groups of cfg->group columns, a power of two in
 * [32, block]; cfg->axis must be CAFEQ_AXIS_COL).  The transform is orthogonal, so
 *   losses[0] = ||Q(Z) - Z||_F^2 = ||M^-1 Q(M W) - W||_F^2 (the l2 proxy),  losses[1] = ||W||_F^2.
 * Z (float32 [rows][cols]), codes, scales: optional outputs, dense.  Workspace:
 * cafeq_hadamard_workspace_bytes(rows, cols, block). */
size_t cafeq_hadamard_workspace_bytes(int64_t rows, int64_t cols, int block);
int cafeq_hadamard_rtn(const cafeq_mat* W, const float* signs, int block, const cafeq_quant_cfg* cfg,
                       float* Z, int8_t* codes, float* scales, float* losses, void* ws, void* stream);

/* Inference side of a single transformed matrix (paper Sec. 4.1, the display Y^ = X M^-1 Q(MW); the
 * block-size table's "extra FLOPs / extra wall-clock time" rows price its first factor).  With the
 * [out][in] layout and Z = W . blockdiag(T) of this library:
 *   x'[t][b*k + i] = sum_j Tinv[b][i][j] X[t][b*k + j],   Y[t][o] = sum_c scales[o][c/group] codes[o][c] x'[t][c].
 * X: float32 [n][in] (leading dimension ldx, a multiple of 4; 16-byte aligned), n >= 1 tokens -- the
 * kernels are laid out for a handful of tokens (the codes are re-read once per 4 tokens);
 * xf: the transform (only Tinv, k, nb are read; nb*k == in, rep == 1), or NULL for the plain quantized
 * layer Y = X Q(W)^T with no transform; codes int8 [out][in] and scales float32 [out][in/group] as
 * written by cafeq_rtn_quantize / cafeq_proxy_loss_fwd_bwd on CAFEQ_AXIS_COL (group 0 = the whole
 * line; in and group multiples of 16, in <= 65536); Y: float32 [n][out] (leading dimension ldy).
 * ws: cafeq_infer_workspace_bytes(n, in) bytes (holds x'; not needed when xf is NULL).
 * float32 accumulation throughout; the summation order is fixed (results are reproducible). */
size_t cafeq_infer_workspace_bytes(int n, int64_t in);
int cafeq_infer_single(const float* X, int n, int64_t ldx, const cafeq_xform* xf, const int8_t* codes,
                       const float* scales, int64_t out, int64_t in, int group, float* Y, int64_t ldy,
                       void* ws, void* stream);

/* Z = W.blockdiag(X) or blockdiag(X).W with X = T (CAFEQ_SIDE_T) or Tinv
 * (CAFEQ_SIDE_TINV)  (paper Sec. 4.1 block-diagonal M; Sec. 4.2 U = W1 M, V = M^-1 W2).
 * Z: float32 [rows][cols] dense, must not alias W. */
int cafeq_apply_transform(const cafeq_mat* W, const cafeq_xform* x, int axis, int side,
                          float* Z, void* ws, void* stream);

/* Prepared weights (see cafeq_mat::prepared).  cafeq_prepared_bytes: size of the buffer for W transformed
 * along `axis` (0 if the axis length is not a multiple of 128); about rows * cols * 8 bytes whatever the
 * storage type: one copy in the order the loss pass contracts (over the axis), one in the order the gradient
 * pass contracts (over the lines; bfloat16 hi + mid parts, tiles of 128 lines x 128 axis indices; read by the
 * gradient pass for blocks of 128 whatever the group and grid).
 * cafeq_prepare_weights fills it (device memory, 256-byte aligned, owned by the caller).  The loss pass's copy:
 * per tile of 32 lines x 128 axis indices two float16 parts of every element -- the line's segment scaled
 * by a power of two so that its largest magnitude lies in [2^3, 2^4), hi = fl16(y), lo = fl16(y - hi):
 * 22 significant bits -- in the order the loss kernel's matrix instructions read them, the per-line
 * factors that undo the scaling, and ||W||_F^2 (float64 sum).  To be called again whenever W changes. */
size_t cafeq_prepared_bytes(const cafeq_mat* W, int axis);
int cafeq_prepare_weights(const cafeq_mat* W, int axis, void* prepared, void* stream);

/* One evaluation for a single matrix (paper Sec. 4 and 4.1), transform along cfg->axis:
 *   Z = transform(W, T); Zq = dequant(Q(Z)); E = Zq - Z; D = transform(E, Tinv)
 *   losses[0] = ||D||_F^2   (= ||M^-1 Q(MW) - W||_F^2, the l2 proxy)
 *   losses[1] = ||E||_F^2
 *   losses[2] = ||W||_F^2
 *   losses[3] = L_sur = beta * sum_G a_G^2 * sum_{j in G} rho_j, beta = 1/(4 qmax^2):
 *               the stochastic-rounding upper bound gradient descent runs on, written
 *               for per-group scales (a_G: group absmax of Z, rho_j: squared norm of the
 *               row (AXIS_COL) / column (AXIS_ROW) j of Tinv)
 *   gradT[nb][k][k] (may be NULL: forward only) = d L_sur / d T with Tinv = T^-1,
 *               absmax differentiated at its arg-max element.
 *   codes / scales (may be NULL): Q(Z) as in cafeq_rtn_quantize.
 * Groups: 32, 64, 128 or 256 elements (max(group, k) must divide the axis), or any longer group that is a
 * multiple of k and divides the axis -- group = 0, the whole channel (the per-channel setting of the paper's
 * experiments, Sec. 6), included.  A group longer than 256 spans several segments of the kernel: the
 * transform is then applied twice (a first sweep finds every group's absmax), and the gradient needs the
 * axis to be a multiple of 128.  Every block size has a gradient for every such group.
 * cfg->mode = CAFEQ_Q_ASYM_MINMAX: Q is the grid of Eq. (1) in the single-precision recipe of
 * cafeq_rtn_quantize_minmax (losses[0], losses[1], codes, scales follow it); L_sur keeps the group absmax
 * and takes the constant the paper prints for that grid, beta = 1/(2^b - 1)^2 (Sec. 4.1); codes are then
 * unsigned bytes in [0, 2^b - 1] and `scales` holds twice as many floats: the scales, then the group minima
 * in the same layout.  On this grid the gradient always runs as the second pass (axis a multiple of 128),
 * and a prepared copy of the weights is ignored. */
int cafeq_proxy_loss_fwd_bwd(const cafeq_mat* W, const cafeq_xform* x,
                             const cafeq_quant_cfg* cfg, float* losses, float* gradT,
                             int8_t* codes, float* scales, void* ws, void* stream);

/* One evaluation for a coupled pair (paper Sec. 4.2): A [d1][nb*k] gets T on its columns
 * (U = A T), B [nb*rep*k][d3] gets Tinv on its rows (V = Tinv B).  cfg->axis is ignored
 * (A is quantized along its columns, B along its rows).
 *   losses[0] = ||Q(U)-U||_F^2      losses[1] = ||Q(V)-V||_F^2
 *   losses[2] = ||Q(U) Tinv - A||_F^2   losses[3] = ||T Q(V) - B||_F^2
 *   losses[4] = LSE = (1/t) log( sum over every group G of U and of V of exp(t a_G) )
 *   losses[5] = number of groups (as float)
 *   gradT[nb][k][k] (may be NULL) = d LSE / d T.
 * codesU/scalesU/codesV/scalesV (may be NULL): Q(U), Q(V).
 * Groups and cfg->mode as in cafeq_proxy_loss_fwd_bwd (with group = 0 the LSE is the paper's sum over the
 * channel maxima m_u(i), m_v(j) of Sec. 4.2; the LSE is a function of the group maxima alone, so the grid
 * changes losses[0..3] and the codes, not losses[4] or gradT). */
int cafeq_dual_proxy_loss_fwd_bwd(const cafeq_mat* A, const cafeq_mat* B,
                                  const cafeq_xform* x, const cafeq_quant_cfg* cfg,
                                  float lse_t, float* losses, float* gradT,
                                  int8_t* codesU, float* scalesU, int8_t* codesV,
                                  float* scalesV, void* ws, void* stream);

/* One iteration of Alg. 1 in transformed coordinates (W1 := U [rowsA][nb*k], float32,
 * W2 := V [nb*rep*k][colsB], float32), per head b (column block b of U, row-blocks
 * q with q / rep == b of V), the pseudoinverse formed from k x k normal equations:
 *   half 0 or 1 (line 3):  Vq <- Q( (Uq^T Uq)^-1 Uq^T U_b . V_q )
 *   half 0 or 2 (line 4):  Uq_b <- Q( U_b . (V_[b] Vq_[b]^T)(Vq_[b] Vq_[b]^T)^-1 )
 * where Uq / Vq are the dequantized current codes (in/out: codesU, scalesU, codesV,
 * scalesV; U groups along columns, V groups along rows).  status[2*nb] (may be NULL):
 * per head and line, 0 ok, 1 the Gram matrix was singular to working precision (a pivot
 * below 1e-5 of its largest entry: the quantized block is rank deficient); that line then
 * falls back to plain rounding of the head's target, i.e. the correction matrix is the
 * identity. */
int cafeq_adaptive_round_step(const float* U, const float* V, int64_t rowsA, int64_t colsA,
                              int64_t rowsB, int64_t colsB, const cafeq_quant_cfg* cfg,
                              int k, int nb, int rep, int half, int8_t* codesU,
                              float* scalesU, int8_t* codesV, float* scalesV, int* status,
                              void* ws, void* stream);

/* Paired quantization error of a transformed pair (paper Sec. 4.2, || W1 W2 - Q(W1) Q(W2) ||_F: the
 * quantity Alg. 1 lowers and the paper's tables on pairs report), per head as in
 * cafeq_adaptive_round_step: with Uq, Vq the dequantized codes,
 *   out[0] = sum over heads b and their row-blocks q of || Uq_b Vq_q - U_b V_q ||_F^2
 *   out[1] = sum of || U_b V_q ||_F^2            (relative PQE = sqrt(out[0] / out[1]))
 * The d1 x d3 products are never formed: both sums are traces of products of k x k Gram
 * matrices of each member (float32 matrix-core sums, float64 from there on), written on the
 * rounding errors so that no large terms cancel. */
int cafeq_pqe(const float* U, const float* V, int64_t rowsA, int64_t colsA, int64_t rowsB,
              int64_t colsB, const cafeq_quant_cfg* cfg, int k, int nb, int rep,
              const int8_t* codesU, const float* scalesU, const int8_t* codesV,
              const float* scalesV, float* out, void* ws, void* stream);

/* ---- Learning the transform ------------------------------------------------------------
 * Paper Sec. 4.1: M is initialised block-diagonal with random rotations and learned by
 * gradient descent on the surrogate; Sec. 4.2 and the appendix on paired-quantization
 * hyperparameters: pairs are learned with Adam on the LogSumExp surrogate, optionally with
 * the regulariser ||T T^T - I||_F / sqrt(d) weighted by lambda_orth. */

/* value[1] (may be NULL) = lambda * ||T T^T - I||_F / sqrt(nb*k), one norm over all blocks.
 * gradT[nb][k][k] (may be NULL) is INCREMENTED by its gradient
 * 2 lambda (T T^T - I) T / (sqrt(nb*k) ||T T^T - I||_F); nothing is added where the norm
 * vanishes.  The residual is formed with float64 accumulation. */
int cafeq_orth_penalty(const float* T, int k, int nb, float lambda, float* value, float* gradT,
                       void* ws, void* stream);

/* T[i] -= lr * grad[i] / *denom for i < n.  denom: device pointer to one float, NULL = 1. */
int cafeq_sgd_update(float* T, const float* grad, float lr, const float* denom, int64_t n,
                     void* stream);

/* One step of Adam with bias correction.  m, v: first / second moment, n floats each, zero
 * before step 1; step counts from 1.  The hyper-parameters are doubles (1 - beta2 is formed
 * in double); the element arithmetic is float32. */
int cafeq_adam_update(float* T, const float* grad, float* m, float* v, int step, double lr,
                      double beta1, double beta2, double eps, int64_t n, void* stream);

typedef struct {
  int steps;          /* iterations */
  float lr;           /* learning rate */
  float lambda_orth;  /* weight of the orthonormality regulariser, 0 = off */
  int normalize;      /* single matrix: divide the surrogate's gradient by ||W||_F^2, so that
                         the loss bounds the squared RELATIVE l2 error and lr is dimensionless */
  double beta1, beta2, eps; /* Adam (pairs) */
} cafeq_opt_cfg;

/* steps iterations of { Tinv = T^-1; losses and gradient at T; + regulariser; T -= update },
 * all enqueued on the stream, no host synchronisation.  T is updated in place; on return
 * (stream order) Tinv is the inverse of the final T and status[nb] (may be NULL) that
 * inversion's status.  history[steps][8] (device): the losses evaluated at the T of each
 * step, before its update:
 *   single: l2_sq, err_z_sq, w_sq, surrogate, penalty, 0, 0, 0     (gradient descent)
 *   pair:   errU_sq, errV_sq, l2A_sq, l2B_sq, lse, n_groups, penalty, 0   (Adam)
 * moments (pair): 2*nb*k*k floats of optimiser state, zeroed by the call. */
int cafeq_optimize_single(const cafeq_mat* W, float* T, float* Tinv, int k, int nb, int rep,
                          const cafeq_quant_cfg* cfg, const cafeq_opt_cfg* opt, float* history,
                          int* status, void* ws, void* stream);
int cafeq_optimize_pair(const cafeq_mat* A, const cafeq_mat* B, float* T, float* Tinv, int k,
                        int nb, int rep, const cafeq_quant_cfg* cfg, float lse_t,
                        const cafeq_opt_cfg* opt, float* moments, float* history, int* status,
                        void* ws, void* stream);

/* Measurement aid (not part of the method).  While a table is installed, every launch of the fused transform
 * kernel (the loss pass; not the gradient pass or the small kernels around it) is bracketed by two of the
 * CALLER's events, recorded on the launch stream: launch number i uses start[i] / stop[i] (hipEvent_t handles
 * the caller created with timing enabled) and count is incremented; launches beyond `capacity` are not
 * timed.  every > 1 times only every `every`-th such launch (an event pair costs the stream several
 * microseconds; `seen` counts all of them and starts at 0).  The library creates, destroys and synchronises nothing: the caller synchronises the stream and reads
 * hipEventElapsedTime(start[i], stop[i]).  The table (host memory) must stay valid until it is replaced or
 * removed with NULL.  One table per process; not thread-safe.
 * kind selects what is timed: 0 the fused transform kernel (the loss pass), 1 the gradient pass over the weights
 * (the second pass of the calls that take the gradient from arg-max records; fused-gradient kernels are kind 0). */
typedef struct {
  void** start;
  void** stop;
  int capacity;
  int count;
  int every;
  int seen;
  int kind;
} cafeq_launch_timing;
int cafeq_set_launch_timing(cafeq_launch_timing* t);

/* Measurement aid (not part of the method): one launch of a plain streaming read over `bytes` bytes of device
 * memory at `buf` (16-byte aligned, bytes a multiple of 16; each lane issues four independent 128-bit loads per
 * step, thousands of small workgroups) -- what the memory system delivers to a kernel that does nothing else,
 * the yardstick for the bandwidth-bound passes.  sink: 4 bytes of device memory that the kernel may write (it
 * writes only if the XOR of everything read equals one particular value).  Enqueued on `stream`; the caller times
 * it.  CAFEQ_ERR_INVALID_ARG for NULL pointers, misalignment or bytes < 16. */
int cafeq_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CAFEQ_H */
