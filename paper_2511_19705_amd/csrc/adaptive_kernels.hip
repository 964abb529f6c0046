// Kernels of the adaptive-rounding step (paper Sec. 5, Alg. 1) in transformed coordinates.
//
// Alg. 1 alternates  W2^ <- Q(pinv(W1^) W1 W2)  and  W1^ <- Q(W1 W2 pinv(W2^)).  Per head the
// pseudoinverse of a full-column-rank (resp. full-row-rank) quantized block is formed from
// k x k normal equations.  With Xq the dequantized codes and E = Xq - X the current rounding
// error, both lines have the same shape:
//     S = Gram(Xq, Xq),  R = Gram(Xq, E),   C = I - S^-1 R
// where Gram(X, Y)[a][b] = sum_t X[t][a] Y[t][b]; t runs over the rows of U (line 3) or over
// the columns of the head's row-blocks of V (line 4), a and b over the k indices of the head.
// Line 3 quantizes C . V_q, line 4 quantizes U_b . C^T (the fused core is handed C as the
// [out][in] operand either way).  Working with E instead of X keeps the float32 Gram sums at
// the scale of the correction, not of the identity it is subtracted from.
//
//   gram_pair_kernel : fp32 MFMA (v_mfma_f32_32x32x2_f32), one workgroup per (head, 32-row
//                      output stripe, chunk of the contraction range); codes are dequantized
//                      on the fly; chunk partials are written out, not atomically added.
//   gj_solve_kernel  : sums the chunk partials in float64 and runs Gauss-Jordan elimination
//                      with partial pivoting on [S | R]; also serves cafeq_block_inverse
//                      ([T | I]).
#include "xform_core.hpp"

namespace cafeq {

namespace {

struct GramArgs {
  const float* X;        // original (transformed) matrix, float32 dense
  const int8_t* codes;   // its current codes
  const float* scales;   // its current scales
  int64_t rows, cols;
  int K, G, rep;
  int64_t tlen;          // contraction length per row-block (rows of U / columns of V)
  int64_t chunk;         // contraction elements per workgroup (multiple of 16)
  int nchunk;            // chunks per row-block
  float* partial;        // [nb][rep*nchunk][2][K][K]
};

// AXIS == COL: t = row i, free index = column;  AXIS == ROW: t = column c, free index = row.
template <int AXIS>
__global__ __launch_bounds__(256) void gram_pair_kernel(const GramArgs a) {
  const int K = a.K, KT = K / 32;
  const int b = blockIdx.x, jt1 = blockIdx.y;
  const int z = blockIdx.z;                      // (row-block within head, chunk)
  const int qi = z / a.nchunk, ch = z % a.nchunk;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ln = lane & 31, h = lane >> 5;
  if (wave >= KT) return;
  const int64_t t0 = int64_t(ch) * a.chunk;
  const int64_t t1 = t0 + a.chunk < a.tlen ? t0 + a.chunk : a.tlen;
  // free-index origin of this head / row-block
  const int64_t f0 = AXIS == CAFEQ_AXIS_COL ? int64_t(b) * K : (int64_t(b) * a.rep + qi) * K;

  floatx16 accS[2], accR[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int v = 0; v < 16; ++v) { accS[u][v] = 0.f; accR[u][v] = 0.f; }
  const int nt2 = (KT - wave + 3) / 4;           // output tiles of this wave: jt2 = wave + 4u

  if (AXIS == CAFEQ_AXIS_COL) {
    const int64_t C = a.cols, SG = a.cols / a.G;
    for (int64_t t = t0; t < t1; t += 16) {
      // eight MFMA steps: step e covers rows t + 2e + h
      float xa[8], xb[2][8], eb[2][8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int64_t i = t + 2 * e + h;
        const bool ok = i < t1;
        const int64_t ca = f0 + jt1 * 32 + ln;
        xa[e] = ok ? __fmul_rn(float(a.codes[i * C + ca]), a.scales[i * SG + ca / a.G]) : 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int64_t cb = f0 + (wave + 4 * u) * 32 + ln;
          if (u < nt2 && ok) {
            const float q = __fmul_rn(float(a.codes[i * C + cb]), a.scales[i * SG + cb / a.G]);
            xb[u][e] = q;
            eb[u][e] = q - a.X[i * C + cb];
          } else {
            xb[u][e] = 0.f; eb[u][e] = 0.f;
          }
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int u = 0; u < 2; ++u)
          if (u < nt2) {
            accS[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e], xb[u][e], accS[u], 0, 0, 0);
            accR[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e], eb[u][e], accR[u], 0, 0, 0);
          }
    }
  } else {
    const int64_t C = a.cols;
    for (int64_t t = t0; t < t1; t += 16) {
      // two groups of four steps: step (g4, e) covers columns t + 8*g4 + 4h + e
      float xa[8], xb[2][8], eb[2][8];
#pragma unroll
      for (int g4 = 0; g4 < 2; ++g4) {
        const int64_t c = t + 8 * g4 + 4 * h;
        const bool ok = c < t1;                   // tlen and chunk are multiples of 4
        const int64_t ra = f0 + jt1 * 32 + ln;
        float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
        uint32_t cw = 0;
        if (ok) {
          s4 = *reinterpret_cast<const float4*>(a.scales + (ra / a.G) * C + c);
          cw = *reinterpret_cast<const uint32_t*>(a.codes + ra * C + c);
        }
        xa[4 * g4 + 0] = __fmul_rn(float(int8_t(cw)), s4.x);
        xa[4 * g4 + 1] = __fmul_rn(float(int8_t(cw >> 8)), s4.y);
        xa[4 * g4 + 2] = __fmul_rn(float(int8_t(cw >> 16)), s4.z);
        xa[4 * g4 + 3] = __fmul_rn(float(int8_t(cw >> 24)), s4.w);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int64_t rb = f0 + (wave + 4 * u) * 32 + ln;
          float4 sb = make_float4(0.f, 0.f, 0.f, 0.f), xv = make_float4(0.f, 0.f, 0.f, 0.f);
          uint32_t cb = 0;
          if (u < nt2 && ok) {
            sb = *reinterpret_cast<const float4*>(a.scales + (rb / a.G) * C + c);
            cb = *reinterpret_cast<const uint32_t*>(a.codes + rb * C + c);
            xv = *reinterpret_cast<const float4*>(a.X + rb * C + c);
          }
          const float q0 = __fmul_rn(float(int8_t(cb)), sb.x), q1 = __fmul_rn(float(int8_t(cb >> 8)), sb.y);
          const float q2 = __fmul_rn(float(int8_t(cb >> 16)), sb.z), q3 = __fmul_rn(float(int8_t(cb >> 24)), sb.w);
          xb[u][4 * g4 + 0] = q0; xb[u][4 * g4 + 1] = q1; xb[u][4 * g4 + 2] = q2; xb[u][4 * g4 + 3] = q3;
          eb[u][4 * g4 + 0] = q0 - xv.x; eb[u][4 * g4 + 1] = q1 - xv.y;
          eb[u][4 * g4 + 2] = q2 - xv.z; eb[u][4 * g4 + 3] = q3 - xv.w;
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int u = 0; u < 2; ++u)
          if (u < nt2) {
            accS[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e], xb[u][e], accS[u], 0, 0, 0);
            accR[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e], eb[u][e], accR[u], 0, 0, 0);
          }
    }
  }

  // partial[b][z][0|1][row][col]
  float* out = a.partial + ((size_t(b) * gridDim.z + z) * 2) * size_t(K) * K;
#pragma unroll
  for (int u = 0; u < 2; ++u)
    if (u < nt2) {
      const int col = (wave + 4 * u) * 32 + ln;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = jt1 * 32 + 8 * (v / 4) + 4 * h + (v % 4);
        out[size_t(row) * K + col] = accS[u][v];
        out[size_t(K) * K + size_t(row) * K + col] = accR[u][v];
      }
    }
}

// Gauss-Jordan on the augmented [A | B] (K x 2K, float64, in `work`), one workgroup per block.
//   mode 0: A = T_b (float32), B = I;            out = A^-1            (block inverse)
//   mode 1: A = sum_z partial S, B = sum_z partial R;  out = I - A^-1 B (adaptive rounding)
// status[b] = 1 when a pivot vanishes to working precision; out is then the identity.
struct GjArgs {
  int mode, K, nz;
  const float* T;        // mode 0
  const float* partial;  // mode 1: [nb][nz][2][K][K]
  double* work;          // [nb][K][2K]
  float* out;            // [nb][K][K]
  float* rho_row; float* rho_col;  // mode 0, optional
  int* status; int status_stride, status_offset;
};
__global__ __launch_bounds__(1024) void gj_solve_kernel(const GjArgs a) {
  __shared__ double pv_val[1024];
  __shared__ int pv_idx[1024];
  __shared__ double prow[512];
  __shared__ double colk[256];
  __shared__ int singular;
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x, K = a.K, W2 = 2 * K;
  double* M = a.work + size_t(b) * K * W2;
  double anorm = 0;
  for (int e = tid; e < K * W2; e += nt) {
    const int r = e / W2, c = e % W2;
    double v;
    if (a.mode == 0) {
      v = c < K ? double(a.T[size_t(b) * K * K + r * K + c]) : (c - K == r ? 1.0 : 0.0);
    } else {
      const float* p = a.partial + size_t(b) * a.nz * 2 * K * K + (c < K ? 0 : size_t(K) * K) + size_t(r) * K + (c % K);
      v = 0;
      for (int z = 0; z < a.nz; ++z) v += double(p[size_t(z) * 2 * K * K]);
    }
    M[e] = v;
    if (c < K) anorm = fmax(anorm, fabs(v));
  }
  pv_val[tid] = anorm;
  if (tid == 0) singular = 0;
  __syncthreads();
  for (int s = nt / 2; s > 0; s >>= 1) {
    if (tid < s) pv_val[tid] = fmax(pv_val[tid], pv_val[tid + s]);
    __syncthreads();
  }
  anorm = pv_val[0];
  __syncthreads();
  for (int k = 0; k < K; ++k) {
    double best = -1.0;
    int bi = k;
    for (int r = k + tid; r < K; r += nt) {
      const double v = fabs(M[r * W2 + k]);
      if (v > best) { best = v; bi = r; }
    }
    pv_val[tid] = best; pv_idx[tid] = bi;
    __syncthreads();
    for (int s = nt / 2; s > 0; s >>= 1) {
      if (tid < s) {
        if (pv_val[tid + s] > pv_val[tid] || (pv_val[tid + s] == pv_val[tid] && pv_idx[tid + s] < pv_idx[tid])) {
          pv_val[tid] = pv_val[tid + s]; pv_idx[tid] = pv_idx[tid + s];
        }
      }
      __syncthreads();
    }
    const int p = pv_idx[0];
    const double pval = pv_val[0];
    __syncthreads();
    // float32-sourced Gram sums carry ~1e-6 relative noise: smaller pivots are not information
    if (!(pval > anorm * (a.mode == 1 ? 1e-5 : 1e-12))) {          // uniform over the workgroup
      if (tid == 0) singular = 1;
      break;
    }
    const double piv = M[p * W2 + k];
    for (int c = tid; c < W2; c += nt) {
      const double vp = M[p * W2 + c], vk = M[k * W2 + c];
      prow[c] = vp / piv;
      if (p != k) M[p * W2 + c] = vk;
    }
    __syncthreads();
    for (int r = tid; r < K; r += nt) colk[r] = (r == k) ? 0.0 : M[r * W2 + k];
    __syncthreads();
    for (int e = tid; e < K * W2; e += nt) {
      const int r = e / W2, c = e % W2;
      M[e] = (r == k) ? prow[c] : M[e] - colk[r] * prow[c];
    }
    __syncthreads();
  }
  __syncthreads();
  const int bad = singular;
  if (a.status && tid == 0) a.status[size_t(b) * a.status_stride + a.status_offset] = bad;
  float* O = a.out + size_t(b) * K * K;
  for (int e = tid; e < K * K; e += nt) {
    const int r = e / K, c = e % K;
    const double x = M[r * W2 + K + c];
    float v;
    if (bad) v = (a.mode == 1 && r == c) ? 1.f : (a.mode == 1 ? 0.f : float(x));
    else v = a.mode == 0 ? float(x) : float((r == c ? 1.0 : 0.0) - x);
    O[e] = v;
  }
  if (a.mode == 0 && (a.rho_row || a.rho_col)) {
    __syncthreads();
    for (int j = tid; j < K; j += nt) {
      double rr = 0, cc = 0;
      for (int i = 0; i < K; ++i) {
        const double x = M[j * W2 + K + i], y = M[i * W2 + K + j];
        rr += x * x; cc += y * y;
      }
      if (a.rho_row) a.rho_row[size_t(b) * K + j] = float(rr);
      if (a.rho_col) a.rho_col[size_t(b) * K + j] = float(cc);
    }
  }
}

}  // namespace

int launch_gram_pair(int axis, const float* X, const int8_t* codes, const float* scales, int64_t rows,
                     int64_t cols, int K, int G, int nb, int rep, int64_t chunk, int nchunk, float* partial,
                     hipStream_t st) {
  GramArgs a;
  a.X = X; a.codes = codes; a.scales = scales; a.rows = rows; a.cols = cols; a.K = K; a.G = G;
  a.rep = axis == CAFEQ_AXIS_COL ? 1 : rep;
  a.tlen = axis == CAFEQ_AXIS_COL ? rows : cols;
  a.chunk = chunk; a.nchunk = nchunk; a.partial = partial;
  dim3 grid(nb, K / 32, a.rep * nchunk);
  if (axis == CAFEQ_AXIS_COL) hipLaunchKernelGGL(gram_pair_kernel<CAFEQ_AXIS_COL>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(gram_pair_kernel<CAFEQ_AXIS_ROW>, grid, dim3(256), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_gj_solve(int K, int nb, int nz, const float* partial, double* work, float* out, int* status,
                    int status_stride, int status_offset, hipStream_t st) {
  GjArgs a;
  a.mode = 1; a.K = K; a.nz = nz; a.T = nullptr; a.partial = partial; a.work = work; a.out = out;
  a.rho_row = a.rho_col = nullptr; a.status = status; a.status_stride = status_stride;
  a.status_offset = status_offset;
  hipLaunchKernelGGL(gj_solve_kernel, dim3(nb), dim3(1024), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_block_inverse(const float* T, int K, int nb, double* work, float* Tinv, float* rho_row,
                         float* rho_col, int* status, hipStream_t st) {
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = 0; a.T = T; a.partial = nullptr; a.work = work; a.out = Tinv;
  a.rho_row = rho_row; a.rho_col = rho_col; a.status = status; a.status_stride = 1; a.status_offset = 0;
  hipLaunchKernelGGL(gj_solve_kernel, dim3(nb), dim3(1024), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // namespace cafeq
