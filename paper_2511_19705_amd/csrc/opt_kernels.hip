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

}  // namespace cafeq

using namespace cafeq;

extern "C" {

int cafeq_orth_penalty(const float* T, int k, int nb, float lambda, float* value, float* gradT, void* ws,
                       void* stream) {
  if (!T || (!value && !gradT)) return CAFEQ_ERR_INVALID_ARG;
  if (nb < 1) return CAFEQ_ERR_BAD_SHAPE;
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
