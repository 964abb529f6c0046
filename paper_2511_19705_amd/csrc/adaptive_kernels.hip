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
#include <type_traits>

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


// Compile-time loop: f(integral_constant<int, I>) for I in [B, E).
template <int B, int E>
struct StaticFor {
  template <typename F>
  static __device__ __forceinline__ void run(F& f) {
    f(std::integral_constant<int, B>{});
    StaticFor<B + 1, E>::run(f);
  }
};
template <int E>
struct StaticFor<E, E> {
  template <typename F>
  static __device__ __forceinline__ void run(F&) {}
};

// Register-resident in-place Gauss-Jordan inversion, one workgroup per block.
// Thread (r, qd) keeps columns [qd*CPT, (qd+1)*CPT) of row r in registers.  Step k: the owners
// of column k publish it, every wave finds the pivot among the rows not yet used (no physical
// row swaps: the pivot order is a permutation undone on output), the pivot row is published
// scaled, and every thread updates its CPT registers -- two barriers per step, and only
// 2K values per step go through LDS.  The step loop is unrolled over the register index so
// that all register accesses are static.
//   A = T_b (float32) when partial == nullptr, else the float64 sum over nz chunk partials
//   of S (first of the two K x K matrices of each partial).  out = A^-1 (zeros if singular).
template <int K, int CPT, typename S>
__global__ __launch_bounds__(K*(K / CPT)) void gj_reg_kernel(const GjArgs a) {
  constexpr int NQ = K / CPT, NTHR = K * NQ, NWAVE = (NTHR + 63) / 64;
  __shared__ S colbuf[2][K];
  __shared__ S rowbuf[2][K];
  __shared__ int pk[K], kinv[K], used[K];
  __shared__ S wred[16];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int r = tid / NQ, qd = tid % NQ;
  S reg[CPT];
  S anorm = 0;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int e = r * K + qd * CPT + j;
    S v;
    if (a.partial == nullptr) {
      v = S(a.T[size_t(b) * K * K + e]);
    } else {
      const float* p = a.partial + size_t(b) * a.nz * 2 * K * K + e;
      double acc = 0;
      for (int z = 0; z < a.nz; ++z) acc += double(p[size_t(z) * 2 * K * K]);
      v = S(acc);
    }
    reg[j] = v;
    anorm = fmax(anorm, fabs(v));
  }
  for (int m = 1; m < 64; m <<= 1) anorm = fmax(anorm, __shfl_xor(anorm, m));
  if (lane == 0) wred[tid >> 6] = anorm;
  if (tid < K) used[tid] = 0;
  __syncthreads();
  anorm = 0;
  for (int i = 0; i < NWAVE; ++i) anorm = fmax(anorm, wred[i]);
  const S tol = anorm * S(a.partial ? 1e-5 : (sizeof(S) == 8 ? 1e-12 : 1e-6));
  bool dead = false;   // uniform over the workgroup

  for (int kb = 0; kb < NQ; ++kb) {
    // one elimination step for column kb*CPT + kk, kk a compile-time register index
    auto step = [&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      const int k = kb * CPT + kk, buf = k & 1;
      if (qd == kb) colbuf[buf][r] = reg[kk];
      __syncthreads();
      if (!dead) {
        S best = -1;
        int bi = K;
        for (int rr = lane; rr < K; rr += 64) {
          const S v = used[rr] ? S(-1) : fabs(colbuf[buf][rr]);
          if (v > best) { best = v; bi = rr; }
        }
        for (int m = 1; m < 64; m <<= 1) {
          const S ob = __shfl_xor(best, m);
          const int oi = __shfl_xor(bi, m);
          if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        if (!(best > tol)) {
          dead = true;
        } else {
          const int p = bi;
          const S ipiv = S(1) / colbuf[buf][p];
          if (r == p) {
#pragma unroll
            for (int j = 0; j < CPT; ++j) {
              const S v = ((qd == kb && j == kk) ? S(1) : reg[j]) * ipiv;
              reg[j] = v;
              rowbuf[buf][qd * CPT + j] = v;
            }
          }
          if (tid == 0) pk[k] = p;
          __syncthreads();
          if (r != p) {
            const S f = colbuf[buf][r];
            if (qd == kb) reg[kk] = 0;
#pragma unroll
            for (int j = 0; j < CPT; ++j) reg[j] -= f * rowbuf[buf][qd * CPT + j];
          }
          if (tid == 0) used[p] = 1;
        }
      }
    };
    StaticFor<0, CPT>::run(step);
  }
  __syncthreads();
  if (a.status && tid == 0) a.status[size_t(b) * a.status_stride + a.status_offset] = dead ? 1 : 0;
  float* O = a.out + size_t(b) * K * K;
  if (dead) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) O[r * K + qd * CPT + j] = 0.f;
    return;
  }
  if (tid < K) kinv[pk[tid]] = tid;
  __syncthreads();
  // register (r, c) is element (kinv[r], pk[c]) of the inverse
  const int orow = kinv[r];
  S rr = 0;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    O[orow * K + pk[qd * CPT + j]] = float(reg[j]);
    rr += reg[j] * reg[j];
  }
  if (a.rho_row || a.rho_col) {
    // squared row norms: sum over this row's NQ threads (adjacent lanes); column norms by atomics in LDS
    for (int m = 1; m < NQ; m <<= 1) rr += __shfl_xor(rr, m);
    if (a.rho_row && qd == 0) a.rho_row[size_t(b) * K + orow] = float(rr);
    if (a.rho_col) {
      __shared__ float cn[K];
      if (tid < K) cn[tid] = 0.f;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < CPT; ++j) atomicAdd(&cn[pk[qd * CPT + j]], float(reg[j] * reg[j]));
      __syncthreads();
      if (tid < K) a.rho_col[size_t(b) * K + tid] = cn[tid];
    }
  }
}

// R_b = float64 sum over the chunk partials of the second matrix of each partial; C_b = I.
__global__ __launch_bounds__(256) void sum_r_init_c_kernel(const float* __restrict__ partial, int nz, int K,
                                                            float* __restrict__ R, float* __restrict__ C) {
  const int b = blockIdx.x;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < K * K; e += gridDim.y * 256) {
    const float* p = partial + size_t(b) * nz * 2 * K * K + size_t(K) * K + e;
    double acc = 0;
    for (int z = 0; z < nz; ++z) acc += double(p[size_t(z) * 2 * K * K]);
    R[size_t(b) * K * K + e] = float(acc);
    C[size_t(b) * K * K + e] = (e / K == e % K) ? 1.f : 0.f;
  }
}


// Float64-accumulating batched product for the iterative refinement of the K = 256 solve:
// C_b (double) = alpha * A_b B_b + beta * C_b, A and B float or double, 64 x 64 tile per workgroup.
template <typename AT, typename BT>
__global__ __launch_bounds__(256) void bgemm_f64acc_kernel(const AT* __restrict__ A, const BT* __restrict__ B,
                                                            double* __restrict__ C, int K, double alpha, double beta) {
  __shared__ double sa[16][66];   // [l][i]
  __shared__ double sb[16][66];   // [l][j]
  const int tpr = K / 64;
  const int b = blockIdx.x / (tpr * tpr), tile = blockIdx.x % (tpr * tpr);
  const int i0 = (tile / tpr) * 64, j0 = (tile % tpr) * 64;
  const AT* Ab = A + size_t(b) * K * K;
  const BT* Bb = B + size_t(b) * K * K;
  double* Cb = C + size_t(b) * K * K;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  double acc[4][4] = {};
  for (int l0 = 0; l0 < K; l0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      sa[e % 16][e / 16] = double(Ab[(i0 + e / 16) * K + l0 + e % 16]);
      sb[e / 64][e % 64] = double(Bb[(l0 + e / 64) * K + j0 + e % 64]);
    }
    __syncthreads();
#pragma unroll
    for (int l = 0; l < 16; ++l) {
      double av[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { av[u] = sa[l][ty * 4 + u]; bv[u] = sb[l][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fma(av[u], bv[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      double* dst = Cb + (i0 + ty * 4 + u) * K + j0 + tx * 4 + v;
      *dst = alpha * acc[u][v] + (beta != 0.0 ? beta * *dst : 0.0);
    }
}

// S64, R64 and a second copy of R64 (the residual's starting value) from the chunk partials.
__global__ __launch_bounds__(256) void sum_partials64_kernel(const float* __restrict__ partial, int nz, int K,
                                                              double* __restrict__ S64, double* __restrict__ R64,
                                                              double* __restrict__ res) {
  const int b = blockIdx.x;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < K * K; e += gridDim.y * 256) {
    const float* p = partial + size_t(b) * nz * 2 * K * K + e;
    double s = 0, r = 0;
    for (int z = 0; z < nz; ++z) {
      s += double(p[size_t(z) * 2 * K * K]);
      r += double(p[size_t(z) * 2 * K * K + size_t(K) * K]);
    }
    S64[size_t(b) * K * K + e] = s;
    R64[size_t(b) * K * K + e] = r;
    res[size_t(b) * K * K + e] = r;
  }
}
__global__ __launch_bounds__(256) void eye64_kernel(double* __restrict__ X, int K, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  const int e = int(i % (int64_t(K) * K));
  X[i] = (e / K == e % K) ? 1.0 : 0.0;
}
__global__ __launch_bounds__(256) void add64_kernel(const double* __restrict__ D, int64_t n, float* __restrict__ X) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) X[i] = float(double(X[i]) + D[i]);
}
__global__ __launch_bounds__(256) void eye_minus_kernel(const double* __restrict__ X, int K, int64_t n,
                                                         float* __restrict__ C) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  const int e = int(i % (int64_t(K) * K));
  C[i] = float(((e / K == e % K) ? 1.0 : 0.0) - X[i]);
}

}  // namespace

namespace {
int launch_gj(const GjArgs& a, int nb, hipStream_t st) {
  switch (a.K) {
    case 32: hipLaunchKernelGGL((gj_reg_kernel<32, 16, double>), dim3(nb), dim3(64), 0, st, a); break;
    case 64: hipLaunchKernelGGL((gj_reg_kernel<64, 32, double>), dim3(nb), dim3(128), 0, st, a); break;
    case 128: hipLaunchKernelGGL((gj_reg_kernel<128, 32, double>), dim3(nb), dim3(512), 0, st, a); break;
    case 256: hipLaunchKernelGGL((gj_reg_kernel<256, 64, float>), dim3(nb), dim3(1024), 0, st, a); break;
    default: hipLaunchKernelGGL(gj_solve_kernel, dim3(nb), dim3(1024), 0, st, a); break;
  }
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
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

// C_b = I - S_b^-1 R_b with S, R the float64 sums of the chunk partials.  Sinv, R: [nb][K][K]
// float32 scratch; work: 4 * nb * K * K doubles.  A singular S_b yields C_b = I and status 1.
// K <= 128: S is inverted in float64.  K == 256: S is inverted in float32 and the solution
// X = S^-1 R gets one step of iterative refinement with float64 residuals.
int launch_gj_solve(int K, int nb, int nz, const float* partial, double* work, float* Sinv, float* R,
                    float* out, int* status, int status_stride, int status_offset, hipStream_t st) {
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = nz; a.T = nullptr; a.partial = partial; a.work = work; a.out = Sinv;
  a.rho_row = a.rho_col = nullptr; a.status = status; a.status_stride = status_stride;
  a.status_offset = status_offset;
  int rc = launch_gj(a, nb, st);
  if (rc) return rc;
  if (K < 256) {
    hipLaunchKernelGGL(sum_r_init_c_kernel, dim3(nb, 16), dim3(256), 0, st, partial, nz, K, R, out);
    CAFEQ_CHECK_LAUNCH();
    return launch_bgemm(false, false, Sinv, R, out, K, nb, -1.f, 1.f, st);
  }
  const size_t mat = size_t(nb) * K * K;
  double *S64 = work, *R64 = work + mat, *res = work + 2 * mat, *X64 = work + 3 * mat;
  const unsigned grid = unsigned(nb) * (K / 64) * (K / 64);
  hipLaunchKernelGGL(sum_partials64_kernel, dim3(nb, 32), dim3(256), 0, st, partial, nz, K, S64, R64, res);
  hipLaunchKernelGGL((bgemm_f64acc_kernel<float, double>), dim3(grid), dim3(256), 0, st, Sinv, R64, X64, K, 1.0, 0.0);
  hipLaunchKernelGGL((bgemm_f64acc_kernel<double, double>), dim3(grid), dim3(256), 0, st, S64, X64, res, K, -1.0, 1.0);
  hipLaunchKernelGGL((bgemm_f64acc_kernel<float, double>), dim3(grid), dim3(256), 0, st, Sinv, res, X64, K, 1.0, 1.0);
  const int64_t n = int64_t(mat);
  hipLaunchKernelGGL(eye_minus_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, X64, K, n, out);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_block_inverse(const float* T, int K, int nb, double* work, float* Tinv, float* rho_row,
                         float* rho_col, int* status, hipStream_t st) {
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = 0; a.T = T; a.partial = nullptr; a.work = work; a.out = Tinv;
  a.rho_row = rho_row; a.rho_col = rho_col; a.status = status; a.status_stride = 1; a.status_offset = 0;
  if (K != 256) return launch_gj(a, nb, st);
  // K == 256 is eliminated in float32; one Newton step X <- X + X (I - T X) with float64
  // residuals brings the result back to float32 rounding accuracy.
  a.rho_row = a.rho_col = nullptr;
  int rc = launch_gj(a, nb, st);
  if (rc) return rc;
  const size_t mat = size_t(nb) * K * K;
  double *res = work, *X64 = work + mat;
  const unsigned grid = unsigned(nb) * (K / 64) * (K / 64);
  const int64_t n = int64_t(mat);
  hipLaunchKernelGGL(eye64_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, res, K, n);
  hipLaunchKernelGGL((bgemm_f64acc_kernel<float, float>), dim3(grid), dim3(256), 0, st, T, Tinv, res, K, -1.0, 1.0);
  hipLaunchKernelGGL((bgemm_f64acc_kernel<float, double>), dim3(grid), dim3(256), 0, st, Tinv, res, X64, K, 1.0, 0.0);
  hipLaunchKernelGGL(add64_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, X64, n, Tinv);
  CAFEQ_CHECK_LAUNCH();
  if (rho_row && (rc = launch_rho(Tinv, K, nb, 1, rho_row, st))) return rc;
  if (rho_col && (rc = launch_rho(Tinv, K, nb, 0, rho_col, st))) return rc;
  return CAFEQ_OK;
}

}  // namespace cafeq
