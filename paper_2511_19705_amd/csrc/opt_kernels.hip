// Learning the transform: orthonormality regulariser and the update rules.
//
//   cafeq_orth_penalty : lambda * ||T T^T - I||_F / sqrt(nb k), one norm over all blocks (the
//                        regulariser of the paper's appendix on paired-quantization
//                        hyperparameters, "Constraints on T"), and its gradient
//                        2 lambda R T / (sqrt(nb k) ||R||_F), R = T T^T - I.  R is formed with
//                        float64 accumulation: near an orthonormal T it is the difference of
//                        two nearly equal matrices, and its direction is what the gradient uses.
//   cafeq_sgd_update   : plain gradient descent (Sec. 4.1: "perform gradient descent with
//                        [the bound] as the loss"), optionally divided by a device scalar.
//   cafeq_adam_update  : Adam with bias correction (the optimiser the appendix uses for pairs).
#include <cmath>

#include "cafeq_internal.hpp"

namespace cafeq {
namespace {

// grid (nb, K*K/256): R_b[i][j] = sum_l T_b[i][l] T_b[j][l] - delta_ij (float64 accumulation,
// stored as float32); partial[b * gridDim.y + y] = sum of R^2 over this workgroup's elements.
__global__ __launch_bounds__(256) void orth_residual_kernel(const float* __restrict__ T, int K, float* __restrict__ R,
                                                             double* __restrict__ partial) {
  __shared__ double red[4];
  const int b = blockIdx.x, e = blockIdx.y * 256 + threadIdx.x;
  const int i = e / K, j = e % K;
  const float* Tb = T + size_t(b) * K * K;
  double acc = 0.0;
  if (e < K * K) {
    const float* ri = Tb + size_t(i) * K;
    const float* rj = Tb + size_t(j) * K;
    for (int l = 0; l < K; l += 4) {
      const float4 a = *reinterpret_cast<const float4*>(ri + l);
      const float4 c = *reinterpret_cast<const float4*>(rj + l);
      acc += double(a.x) * double(c.x) + double(a.y) * double(c.y) + double(a.z) * double(c.z) +
             double(a.w) * double(c.w);
    }
    acc -= (i == j) ? 1.0 : 0.0;
    R[size_t(b) * K * K + e] = float(acc);
  }
  double sq = acc * acc;
  for (int m = 1; m < 64; m <<= 1) sq += __shfl_xor(sq, m);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
  __syncthreads();
  if (threadIdx.x == 0) partial[size_t(b) * gridDim.y + blockIdx.y] = (red[0] + red[1]) + (red[2] + red[3]);
}

// one workgroup: n = sqrt(sum of the partials in fixed order); value = lambda n / sqrt(d);
// coef = 2 lambda / (sqrt(d) n), or 0 where the norm vanishes
__global__ __launch_bounds__(256) void orth_finish_kernel(const double* __restrict__ partial, int npart, float lambda,
                                                           double d, float* __restrict__ value,
                                                           float* __restrict__ coef) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < npart; i += 256) s += partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int m = 128; m > 0; m >>= 1) {
    if (threadIdx.x < m) red[threadIdx.x] += red[threadIdx.x + m];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double n = sqrt(red[0]);
    if (value) *value = float(double(lambda) * n / sqrt(d));
    *coef = n > 1e-30 ? float(2.0 * double(lambda) / (sqrt(d) * n)) : 0.f;
  }
}

__global__ __launch_bounds__(256) void axpy_dev_kernel(float* __restrict__ y, const float* __restrict__ x,
                                                        const float* __restrict__ coef, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) y[i] += *coef * x[i];
}

__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ T, const float* __restrict__ g, float lr,
                                                   const float* __restrict__ denom, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  const float step = denom ? lr / *denom : lr;
  T[i] -= step * g[i];
}

__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ T, const float* __restrict__ g,
                                                    float* __restrict__ m, float* __restrict__ v, float lr,
                                                    float beta1, float omb1, float beta2, float omb2, float eps,
                                                    float c1, float c2, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  const float gi = g[i];
  const float mi = beta1 * m[i] + omb1 * gi;   // omb = 1 - beta, formed in double on the host
  const float vi = beta2 * v[i] + omb2 * gi * gi;
  m[i] = mi;
  v[i] = vi;
  // c1 = 1 / (1 - beta1^t), c2 = 1 / (1 - beta2^t)
  T[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);
}

__global__ __launch_bounds__(256) void div_dev_kernel(float* __restrict__ g, const float* __restrict__ denom, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) g[i] = g[i] / *denom;
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ p, float value, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = value;
}

}  // namespace

int launch_fill(float* p, float value, int64_t n, hipStream_t st) {
  if (n <= 0) return CAFEQ_OK;
  hipLaunchKernelGGL(fill_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, p, value, n);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_div_by_device_scalar(float* g, const float* denom, int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(div_dev_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, g, denom, n);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

size_t orth_workspace_bytes(int k, int nb) {
  const size_t kk = size_t(nb) * k * k;
  return align_up(kk * sizeof(float), 256) * 2 + align_up(size_t(nb) * ((size_t(k) * k + 255) / 256) * sizeof(double), 256) +
         256;
}


// ---------------------------------------------------------------------------------------------------
// Transform blocks smaller than 32 (the paper's block-size sweep goes down to 2): a run of 32 / k consecutive
// k x k blocks IS one 32 x 32 block that happens to be block-diagonal, so every kernel written for blocks of 32
// serves them.  embed: T32[Q] = blockdiag_i( T[(Q m + i) / rep] ), m = 32 / k (blocks past the end: identity);
// gather: G[b] = sum over the positions block b was placed at of the k x k diagonal sub-block there (chain rule:
// the entries outside the diagonal sub-blocks are derivatives with respect to entries that stay zero), in the
// fixed order of the positions.
namespace {
__global__ __launch_bounds__(256) void embed_blocks_kernel(const float* __restrict__ T, int k, int nb, int rep, int nb32,
                                                            float* __restrict__ T32) {
  const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (e >= int64_t(nb32) * 1024) return;
  const int Q = int(e >> 10), r = int(e >> 5) & 31, c = int(e) & 31;
  const int m = 32 / k, i = r / k;
  float v = 0.f;
  if (c / k == i) {
    const int64_t sb = (int64_t(Q) * m + i) / rep;
    v = sb < nb ? T[(sb * k + r % k) * k + c % k] : (r == c ? 1.f : 0.f);
  }
  T32[e] = v;
}
__global__ __launch_bounds__(256) void gather_blocks_kernel(const float* __restrict__ G32, int k, int nb, int rep,
                                                             float* __restrict__ G) {
  const int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (e >= int64_t(nb) * k * k) return;
  const int b = int(e / (k * k)), r = int(e / k) % k, c = int(e % k);
  const int m = 32 / k;
  float acc = 0.f;
  for (int j = 0; j < rep; ++j) {
    const int64_t q = int64_t(b) * rep + j;
    const int64_t Q = q / m;
    const int i = int(q % m);
    acc += G32[(Q * 32 + i * k + r) * 32 + i * k + c];
  }
  G[e] = acc;
}
}  // namespace

namespace {
__global__ __launch_bounds__(256) void axpy_kernel(float* __restrict__ y, const float* __restrict__ x, float alpha, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) y[i] += alpha * x[i];
}
}  // namespace
int launch_axpy(float* y, const float* x, float alpha, int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(axpy_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, y, x, alpha, n);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
namespace {
__global__ __launch_bounds__(256) void expand_status_kernel(const int* __restrict__ st32, int m, int nb, int* __restrict__ status) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b < nb) status[b] = st32[b / m];
}
}  // namespace
int launch_expand_status(const int* st32, int m, int nb, int* status, hipStream_t st) {
  hipLaunchKernelGGL(expand_status_kernel, dim3(unsigned((nb + 255) / 256)), dim3(256), 0, st, st32, m, nb, status);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_embed_blocks(const float* T, int k, int nb, int rep, int nb32, float* T32, hipStream_t st) {
  const int64_t n = int64_t(nb32) * 1024;
  hipLaunchKernelGGL(embed_blocks_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, T, k, nb, rep, nb32, T32);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_gather_blocks(const float* G32, int k, int nb, int rep, float* G, hipStream_t st) {
  const int64_t n = int64_t(nb) * k * k;
  hipLaunchKernelGGL(gather_blocks_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, G32, k, nb, rep, G);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // namespace cafeq

using namespace cafeq;

extern "C" {

int cafeq_orth_penalty(const float* T, int k, int nb, float lambda, float* value, float* gradT, void* ws,
                       void* stream) {
  if (!T || (!value && !gradT)) return CAFEQ_ERR_INVALID_ARG;
  if (nb < 1) return CAFEQ_ERR_BAD_SHAPE;
  if (k == 2 || k == 4 || k == 8 || k == 16) {
    // a run of 32 / k blocks as one block-diagonal block of 32: T T^T - I keeps its Frobenius norm and d = nb k;
    // the gradient is gathered from the diagonal sub-blocks and ADDED, as for the larger blocks
    const int m = 32 / k;
    if (nb % m != 0) return CAFEQ_ERR_BAD_SHAPE;
    if (!ws) return CAFEQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nb32 = nb / m;
    const size_t blk = align_up(size_t(nb32) * 1024 * sizeof(float), 256);
    char* base = static_cast<char*>(ws);
    float* T32 = reinterpret_cast<float*>(base);
    float* G32 = reinterpret_cast<float*>(base + blk);
    float* Gs = reinterpret_cast<float*>(base + 2 * blk);   // gathered gradient [nb][k][k]
    void* sub = base + 3 * blk + align_up(size_t(nb32) * sizeof(int), 256);
    int rc;
    if ((rc = launch_embed_blocks(T, k, nb, 1, nb32, T32, st))) return rc;
    if (gradT && (rc = launch_fill(G32, 0.f, int64_t(nb32) * 1024, st))) return rc;
    if ((rc = cafeq_orth_penalty(T32, 32, nb32, lambda, value, gradT ? G32 : nullptr, sub, stream))) return rc;
    if (gradT) {
      if ((rc = launch_gather_blocks(G32, k, nb, 1, Gs, st))) return rc;
      if ((rc = launch_axpy(gradT, Gs, 1.f, int64_t(nb) * k * k, st))) return rc;
    }
    return CAFEQ_OK;
  }
  if (k != 32 && k != 64 && k != 128 && k != 256) return CAFEQ_ERR_UNSUPPORTED;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t kk = size_t(nb) * k * k;
  char* base = static_cast<char*>(ws);
  float* R = reinterpret_cast<float*>(base);
  float* G = reinterpret_cast<float*>(base + align_up(kk * sizeof(float), 256));
  const int ny = (k * k + 255) / 256;
  double* partial = reinterpret_cast<double*>(base + 2 * align_up(kk * sizeof(float), 256));
  float* coef = reinterpret_cast<float*>(base + 2 * align_up(kk * sizeof(float), 256) +
                                         align_up(size_t(nb) * ny * sizeof(double), 256));
  hipLaunchKernelGGL(orth_residual_kernel, dim3(nb, ny), dim3(256), 0, st, T, k, R, partial);
  CAFEQ_CHECK_LAUNCH();
  hipLaunchKernelGGL(orth_finish_kernel, dim3(1), dim3(256), 0, st, partial, nb * ny, lambda, double(nb) * k, value,
                     coef);
  CAFEQ_CHECK_LAUNCH();
  if (gradT) {
    int rc = launch_bgemm(false, false, R, T, G, k, nb, 1.f, 0.f, st);
    if (rc) return rc;
    hipLaunchKernelGGL(axpy_dev_kernel, dim3(unsigned((kk + 255) / 256)), dim3(256), 0, st, gradT, G, coef, int64_t(kk));
    CAFEQ_CHECK_LAUNCH();
  }
  return CAFEQ_OK;
}

int cafeq_sgd_update(float* T, const float* grad, float lr, const float* denom, int64_t n, void* stream) {
  if (!T || !grad) return CAFEQ_ERR_INVALID_ARG;
  if (n < 1) return CAFEQ_ERR_BAD_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(sgd_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, T, grad, lr, denom, n);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int cafeq_adam_update(float* T, const float* grad, float* m, float* v, int step, double lr, double beta1, double beta2,
                      double eps, int64_t n, void* stream) {
  if (!T || !grad || !m || !v) return CAFEQ_ERR_INVALID_ARG;
  if (n < 1 || step < 1) return CAFEQ_ERR_BAD_SHAPE;
  if (!(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0)) return CAFEQ_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const float c1 = float(1.0 / (1.0 - pow(beta1, double(step))));
  const float c2 = float(1.0 / (1.0 - pow(beta2, double(step))));
  hipLaunchKernelGGL(adam_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, T, grad, m, v, float(lr),
                     float(beta1), float(1.0 - beta1), float(beta2), float(1.0 - beta2), float(eps), c1, c2, n);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // extern "C"
