// The paper's "random" comparison (caption of the block-size table, Sec. 4.1): a block-diagonal
// transform whose blocks are randomized Hadamard matrices -- random signs, then the normalised
// Walsh-Hadamard transform of each block of 256 / 512 / 1024 consecutive inputs -- followed by
// the symmetric absmax round-to-nearest of cafeq_rtn_quantize.  The transform is orthogonal, so
// the l2 proxy ||M^-1 Q(M W) - W||_F equals the rounding error ||Q(Z) - Z||_F and no way back
// is computed.
//
// One wave owns one (row, block): lane i holds elements 4i .. 4i+3 of each 256-element quarter j
// (one 128-bit load each).  The butterflies over index bits 0-1 and 8-9 stay in registers, bits
// 2-7 go through cross-lane exchanges; then the group absmax (a cluster of g/4 lanes, as in the
// plain kernel), codes, scales and the error sum.  HBM-bound: 4 B read, 1 B (+ 4 B for Z) written
// per element.
#include "cafeq_common.hpp"
#include "cafeq_internal.hpp"

namespace cafeq {
namespace {

struct HadArgs {
  const void* W;
  int64_t rows, cols, ld;
  const float* signs;
  float norm;          // 1 / sqrt(block)
  QGrid grid;
  float* Z;
  uint32_t* codes;
  float* scales;
  double* partial;     // [workgroups][2]: error sum, sum of squares of W
};

// NJ: 256-element quarters per block; LPG: lanes per group inside a quarter; JG: quarters per group
template <typename Tag, int NJ, int LPG, int JG>
__global__ __launch_bounds__(256) void hadamard_rtn_kernel(const HadArgs a) {
  using E = typename Tag::elem;
  constexpr int BLK = 256 * NJ;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t nblk = a.cols / BLK;
  const int64_t task = int64_t(blockIdx.x) * 4 + wave;
  const bool live = task < a.rows * nblk;
  const int64_t row = live ? task / nblk : 0, bk = live ? task - row * nblk : 0;
  const E* src = static_cast<const E*>(a.W) + row * a.ld + bk * BLK + 4 * lane;
  const float* sg = a.signs + bk * BLK + 4 * lane;
  float4 x[NJ];
  float wsq = 0.f;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    x[j] = live ? load4(src + 256 * j) : make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 s = *reinterpret_cast<const float4*>(sg + 256 * j);
    wsq += x[j].x * x[j].x + x[j].y * x[j].y + x[j].z * x[j].z + x[j].w * x[j].w;
    x[j].x *= s.x; x[j].y *= s.y; x[j].z *= s.z; x[j].w *= s.w;
  }
  // ---- index bits 0 and 1: inside the lane's four elements
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const float a0 = x[j].x + x[j].y, a1 = x[j].x - x[j].y, a2 = x[j].z + x[j].w, a3 = x[j].z - x[j].w;
    x[j] = make_float4(a0 + a2, a1 + a3, a0 - a2, a1 - a3);
  }
  // ---- index bits 2..7: the lane index
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const bool up = (lane & m) != 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const float vx = __shfl_xor(x[j].x, m), vy = __shfl_xor(x[j].y, m);
      const float vz = __shfl_xor(x[j].z, m), vw = __shfl_xor(x[j].w, m);
      x[j].x = up ? vx - x[j].x : x[j].x + vx;
      x[j].y = up ? vy - x[j].y : x[j].y + vy;
      x[j].z = up ? vz - x[j].z : x[j].z + vz;
      x[j].w = up ? vw - x[j].w : x[j].w + vw;
    }
  }
  // ---- index bits 8 and 9: across the quarters
#pragma unroll
  for (int m = 1; m < NJ; m <<= 1)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      if ((j & m) == 0) {
        const float4 p = x[j], q = x[j | m];
        x[j] = make_float4(p.x + q.x, p.y + q.y, p.z + q.z, p.w + q.w);
        x[j | m] = make_float4(p.x - q.x, p.y - q.y, p.z - q.z, p.w - q.w);
      }
#pragma unroll
  for (int j = 0; j < NJ; ++j) { x[j].x *= a.norm; x[j].y *= a.norm; x[j].z *= a.norm; x[j].w *= a.norm; }

  // ---- per-group absmax, codes, error
  float am[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    am[j] = fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w)));
    am[j] = cluster_allmax<LPG>(am[j]);
  }
  if constexpr (JG > 1) {
#pragma unroll
    for (int j0 = 0; j0 < NJ; j0 += JG) {
      float m = am[j0];
#pragma unroll
      for (int u = 1; u < JG; ++u) m = fmaxf(m, am[j0 + u]);
#pragma unroll
      for (int u = 0; u < JG; ++u) am[j0 + u] = m;
    }
  }
  float err = 0.f;
  const int64_t e0 = row * a.cols + bk * BLK + 4 * lane;          // element offset (dense outputs)
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const float inv = grid_inv(am[j], a.grid.qmax), s = grid_scale(am[j], a.grid.qmax);
    const float q0 = grid_code(x[j].x, inv, a.grid), q1 = grid_code(x[j].y, inv, a.grid);
    const float q2 = grid_code(x[j].z, inv, a.grid), q3 = grid_code(x[j].w, inv, a.grid);
    const float d0 = __fmul_rn(q0, s) - x[j].x, d1 = __fmul_rn(q1, s) - x[j].y;
    const float d2 = __fmul_rn(q2, s) - x[j].z, d3 = __fmul_rn(q3, s) - x[j].w;
    err += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
    if (live) {
      if (a.Z) *reinterpret_cast<float4*>(a.Z + e0 + 256 * j) = x[j];
      if (a.codes) a.codes[(e0 + 256 * j) / 4] = pack4(q0, q1, q2, q3);
      if (a.scales) {
        constexpr int G = 4 * LPG * JG;
        const bool first = (lane % LPG) == 0 && (j % JG) == 0;
        if (first) a.scales[(e0 + 256 * j) / G] = s;
      }
    }
  }
  if (!live) { err = 0.f; wsq = 0.f; }
  // ---- per-workgroup partials in float64, fixed order
  __shared__ double red[2][4];
  const double de = wave_sum(double(err)), dw = wave_sum(double(wsq));
  if (lane == 0) { red[0][wave] = de; red[1][wave] = dw; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a.partial[2 * size_t(blockIdx.x)] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    a.partial[2 * size_t(blockIdx.x) + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

__global__ __launch_bounds__(256) void hadamard_finish_kernel(const double* __restrict__ partial, int n,
                                                               float* __restrict__ losses) {
  __shared__ double red[2][256];
  double e = 0, w = 0;
  for (int i = threadIdx.x; i < n; i += 256) { e += partial[2 * size_t(i)]; w += partial[2 * size_t(i) + 1]; }
  red[0][threadIdx.x] = e; red[1][threadIdx.x] = w;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) { red[0][threadIdx.x] += red[0][threadIdx.x + s]; red[1][threadIdx.x] += red[1][threadIdx.x + s]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { losses[0] = float(red[0][0]); losses[1] = float(red[1][0]); }
}

template <typename Tag, int NJ>
int launch_had_nj(const HadArgs& a, int g, unsigned nwg, hipStream_t st) {
#define CAFEQ_HAD(LPG, JG) hipLaunchKernelGGL((hadamard_rtn_kernel<Tag, NJ, LPG, JG>), dim3(nwg), dim3(256), 0, st, a)
  switch (g) {
    case 32: CAFEQ_HAD(8, 1); break;
    case 64: CAFEQ_HAD(16, 1); break;
    case 128: CAFEQ_HAD(32, 1); break;
    case 256: CAFEQ_HAD(64, 1); break;
    case 512: if constexpr (NJ >= 2) { CAFEQ_HAD(64, 2); break; } else return CAFEQ_ERR_UNSUPPORTED;
    case 1024: if constexpr (NJ >= 4) { CAFEQ_HAD(64, 4); break; } else return CAFEQ_ERR_UNSUPPORTED;
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
#undef CAFEQ_HAD
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

template <typename Tag>
int launch_had_typed(const HadArgs& a, int block, int g, unsigned nwg, hipStream_t st) {
  switch (block) {
    case 256: return launch_had_nj<Tag, 1>(a, g, nwg, st);
    case 512: return launch_had_nj<Tag, 2>(a, g, nwg, st);
    case 1024: return launch_had_nj<Tag, 4>(a, g, nwg, st);
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
}

}  // namespace
}  // namespace cafeq

using namespace cafeq;

extern "C" {

size_t cafeq_hadamard_workspace_bytes(int64_t rows, int64_t cols, int block) {
  if (rows < 1 || cols < 1 || block < 256) return 0;
  const int64_t tasks = rows * (cols / block);
  return align_up(size_t((tasks + 3) / 4) * 2 * sizeof(double), 256);
}

int cafeq_hadamard_rtn(const cafeq_mat* W, const float* signs, int block, const cafeq_quant_cfg* cfg, float* Z,
                       int8_t* codes, float* scales, float* losses, void* ws, void* stream) {
  if (!W || !W->data || !signs || !cfg || !losses) return CAFEQ_ERR_INVALID_ARG;
  if (W->dtype != CAFEQ_F32 && W->dtype != CAFEQ_BF16) return CAFEQ_ERR_INVALID_ARG;
  if (W->rows < 1 || W->cols < 1 || W->ld < W->cols) return CAFEQ_ERR_BAD_SHAPE;
  if (cfg->axis != CAFEQ_AXIS_COL) return CAFEQ_ERR_UNSUPPORTED;      // blocks run along the contiguous axis
  if (cfg->bits < 2 || cfg->bits > 8) return CAFEQ_ERR_INVALID_ARG;
  if (block != 256 && block != 512 && block != 1024) return CAFEQ_ERR_UNSUPPORTED;
  if (W->cols % block != 0) return CAFEQ_ERR_BAD_SHAPE;
  const int g = cfg->group;
  if (g < 32 || g > block || (g & (g - 1)) != 0) return CAFEQ_ERR_UNSUPPORTED;
  const int64_t ldm = W->dtype == CAFEQ_F32 ? 4 : 8;
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (W->ld % ldm != 0 || !al16(W->data) || !al16(signs) || (Z && !al16(Z)) || (codes && !al16(codes)) ||
      (scales && !al16(scales)))
    return CAFEQ_ERR_BAD_ALIGN;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  HadArgs a;
  a.W = W->data; a.rows = W->rows; a.cols = W->cols; a.ld = W->ld; a.signs = signs;
  a.norm = float(1.0 / sqrt(double(block)));
  a.grid = make_grid(cfg->bits);
  a.Z = Z; a.codes = reinterpret_cast<uint32_t*>(codes); a.scales = scales;
  a.partial = static_cast<double*>(ws);
  const int64_t tasks = W->rows * (W->cols / block);
  const unsigned nwg = unsigned((tasks + 3) / 4);
  int rc = W->dtype == CAFEQ_BF16 ? launch_had_typed<BF16Tag>(a, block, g, nwg, st)
                                  : launch_had_typed<F32Tag>(a, block, g, nwg, st);
  if (rc) return rc;
  hipLaunchKernelGGL(hadamard_finish_kernel, dim3(1), dim3(256), 0, st, a.partial, int(nwg), losses);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // extern "C"
