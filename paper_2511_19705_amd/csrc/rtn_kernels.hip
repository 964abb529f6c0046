// Per-group absmax round-to-nearest without a transform (the HBM-bound stage).
//
// Rounding rule of the paper's Eq. (1) (nearest integer) on the symmetric grid
// described in cafeq.h.  Algorithmic traffic per element: one read (4 B float32 /
// 2 B bfloat16), one int8 code written, 4/g bytes of scale.
//
// Four kernels:
//   rtn_col_fast : groups along the contiguous axis, g = 4 * 2^n <= 256.  One lane owns
//                  four consecutive elements (one 128-bit load), g/4 adjacent lanes own a
//                  group; the absmax is an all-reduce over that lane cluster with DPP
//                  (inside a 16-lane row) and LDS-crossbar shuffles (across rows).
//   rtn_row_fast : groups along the strided axis, g = 16 * {1,2,4,8,16}.  A workgroup of
//                  g/16 waves owns g rows x 256 columns; each wave keeps 16 rows of four
//                  columns per lane in registers, column maxima are combined through LDS,
//                  so the tile is read from memory once.
//   rtn_col_any / rtn_row_any : any group length dividing the line, two passes per group.
// The squared-error output is reduced in two fixed-order stages (per-workgroup partials
// in the caller's workspace, then one workgroup), so it is reproducible run to run.
#include "cafeq_common.hpp"
#include "cafeq_internal.hpp"

namespace cafeq {

namespace {

constexpr int kColThreads = 256;
constexpr int kColUnroll = 4;

__device__ __forceinline__ void block_store_partial(float err, double* partial) {
  __shared__ double red[16];
  double e = wave_sum(double(err));
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (lane == 0) red[wave] = e;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0;
    const int nw = (blockDim.x + kWave - 1) / kWave;
    for (int i = 0; i < nw; ++i) t += red[i];
    partial[blockIdx.y * size_t(gridDim.x) + blockIdx.x] = t;
  }
}

template <typename Tag, int LPG, bool DENSE>
__global__ __launch_bounds__(kColThreads) void rtn_col_fast(
    const typename Tag::elem* __restrict__ W, uint32_t nvec, uint32_t cols4, int64_t ld, QGrid grid,
    uint32_t* __restrict__ codes, float* __restrict__ scales, double* __restrict__ partial) {
  const uint32_t base = blockIdx.x * (kColThreads * kColUnroll) + threadIdx.x;
  float4 x[kColUnroll];
  bool live[kColUnroll];
#pragma unroll
  for (int j = 0; j < kColUnroll; ++j) {
    const uint32_t v = base + j * kColThreads;
    live[j] = v < nvec;
    x[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live[j]) {
      size_t off;
      if constexpr (DENSE) {
        off = size_t(v) * 4;
      } else {
        const uint32_t r = v / cols4;
        off = size_t(r) * ld + size_t(v - r * cols4) * 4;
      }
      x[j] = load4(W + off);
    }
  }
  float err = 0.f;
#pragma unroll
  for (int j = 0; j < kColUnroll; ++j) {
    const uint32_t v = base + j * kColThreads;
    float a = fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w)));
    a = cluster_allmax<LPG>(a);   // executed by every lane: clusters never straddle `live`
    const float inv = grid_inv(a, grid.qmax);
    const float s = grid_scale(a, grid.qmax);
    const float q0 = grid_code(x[j].x, inv, grid), q1 = grid_code(x[j].y, inv, grid);
    const float q2 = grid_code(x[j].z, inv, grid), q3 = grid_code(x[j].w, inv, grid);
    if (live[j]) {
      codes[v] = pack4(q0, q1, q2, q3);
      if ((threadIdx.x % LPG) == 0 && scales) scales[v / LPG] = s;
      if (partial) {
        const float e0 = __fmul_rn(q0, s) - x[j].x, e1 = __fmul_rn(q1, s) - x[j].y;
        const float e2 = __fmul_rn(q2, s) - x[j].z, e3 = __fmul_rn(q3, s) - x[j].w;
        err += e0 * e0 + e1 * e1 + e2 * e2 + e3 * e3;
      }
    }
  }
  if (partial) block_store_partial(err, partial);
}

constexpr int kRowRPW = 16;  // rows per wave

template <typename Tag, int NW>
__global__ __launch_bounds__(NW * kWave) void rtn_row_fast(
    const typename Tag::elem* __restrict__ W, int64_t cols, int64_t ld, QGrid grid,
    int8_t* __restrict__ codes, float* __restrict__ scales, double* __restrict__ partial) {
  __shared__ float4 smax[NW][kWave];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int64_t c = int64_t(blockIdx.x) * 256 + lane * 4;
  const int64_t r0 = int64_t(blockIdx.y) * (NW * kRowRPW) + wave * kRowRPW;
  const bool live = c < cols;
  float4 x[kRowRPW];
  float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int i = 0; i < kRowRPW; ++i) {
    x[i] = live ? load4(W + (r0 + i) * ld + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    m.x = fmaxf(m.x, fabsf(x[i].x));
    m.y = fmaxf(m.y, fabsf(x[i].y));
    m.z = fmaxf(m.z, fabsf(x[i].z));
    m.w = fmaxf(m.w, fabsf(x[i].w));
  }
  if constexpr (NW > 1) {
    smax[wave][lane] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float4 o = smax[w][lane];
      m.x = fmaxf(m.x, o.x);
      m.y = fmaxf(m.y, o.y);
      m.z = fmaxf(m.z, o.z);
      m.w = fmaxf(m.w, o.w);
    }
  }
  const float4 inv = make_float4(grid_inv(m.x, grid.qmax), grid_inv(m.y, grid.qmax),
                                 grid_inv(m.z, grid.qmax), grid_inv(m.w, grid.qmax));
  const float4 s = make_float4(grid_scale(m.x, grid.qmax), grid_scale(m.y, grid.qmax),
                               grid_scale(m.z, grid.qmax), grid_scale(m.w, grid.qmax));
  float err = 0.f;
  if (live) {
    if (wave == 0 && scales) *reinterpret_cast<float4*>(scales + int64_t(blockIdx.y) * cols + c) = s;
#pragma unroll
    for (int i = 0; i < kRowRPW; ++i) {
      const float q0 = grid_code(x[i].x, inv.x, grid), q1 = grid_code(x[i].y, inv.y, grid);
      const float q2 = grid_code(x[i].z, inv.z, grid), q3 = grid_code(x[i].w, inv.w, grid);
      *reinterpret_cast<uint32_t*>(codes + (r0 + i) * cols + c) = pack4(q0, q1, q2, q3);
      if (partial) {
        const float e0 = __fmul_rn(q0, s.x) - x[i].x, e1 = __fmul_rn(q1, s.y) - x[i].y;
        const float e2 = __fmul_rn(q2, s.z) - x[i].z, e3 = __fmul_rn(q3, s.w) - x[i].w;
        err += e0 * e0 + e1 * e1 + e2 * e2 + e3 * e3;
      }
    }
  }
  if (partial) block_store_partial(err, partial);
}

// One wave per group, group length a multiple of 4: 128-bit loads, four codes per store.
template <typename Tag>
__global__ __launch_bounds__(256) void rtn_col_vec(
    const typename Tag::elem* __restrict__ W, int64_t rows, int64_t cols, int64_t ld, int64_t g,
    QGrid grid, int8_t* __restrict__ codes, float* __restrict__ scales, double* __restrict__ partial) {
  const int lane = threadIdx.x % kWave;
  const int64_t gpr = cols / g, ngroups = rows * gpr;
  const int64_t wave0 = int64_t(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t wstride = int64_t(gridDim.x) * (blockDim.x / kWave);
  float err = 0.f;
  for (int64_t gi = wave0; gi < ngroups; gi += wstride) {
    const int64_t r = gi / gpr, c0 = (gi - r * gpr) * g;
    const typename Tag::elem* src = W + r * ld + c0;
    float a = 0.f;
    for (int64_t i = int64_t(lane) * 4; i < g; i += kWave * 4) {
      const float4 z = load4(src + i);
      a = fmaxf(a, fmaxf(fmaxf(fabsf(z.x), fabsf(z.y)), fmaxf(fabsf(z.z), fabsf(z.w))));
    }
    a = cluster_allmax<64>(a);
    const float inv = grid_inv(a, grid.qmax), s = grid_scale(a, grid.qmax);
    if (lane == 0 && scales) scales[gi] = s;
    for (int64_t i = int64_t(lane) * 4; i < g; i += kWave * 4) {
      const float4 z = load4(src + i);
      const float q0 = grid_code(z.x, inv, grid), q1 = grid_code(z.y, inv, grid);
      const float q2 = grid_code(z.z, inv, grid), q3 = grid_code(z.w, inv, grid);
      *reinterpret_cast<uint32_t*>(codes + r * cols + c0 + i) = pack4(q0, q1, q2, q3);
      if (partial) {
        const float e0 = __fmul_rn(q0, s) - z.x, e1 = __fmul_rn(q1, s) - z.y;
        const float e2 = __fmul_rn(q2, s) - z.z, e3 = __fmul_rn(q3, s) - z.w;
        err += e0 * e0 + e1 * e1 + e2 * e2 + e3 * e3;
      }
    }
  }
  if (partial) block_store_partial(err, partial);
}

// One wave per group, any group length.
template <typename Tag>
__global__ __launch_bounds__(256) void rtn_col_any(
    const typename Tag::elem* __restrict__ W, int64_t rows, int64_t cols, int64_t ld, int64_t g,
    QGrid grid, int8_t* __restrict__ codes, float* __restrict__ scales, double* __restrict__ partial) {
  const int lane = threadIdx.x % kWave;
  const int64_t gpr = cols / g, ngroups = rows * gpr;
  const int64_t wave0 = int64_t(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t wstride = int64_t(gridDim.x) * (blockDim.x / kWave);
  float err = 0.f;
  for (int64_t gi = wave0; gi < ngroups; gi += wstride) {
    const int64_t r = gi / gpr, c0 = (gi - r * gpr) * g;
    const typename Tag::elem* src = W + r * ld + c0;
    float a = 0.f;
    for (int64_t i = lane; i < g; i += kWave) a = fmaxf(a, fabsf(load1(src + i)));
    a = cluster_allmax<64>(a);
    const float inv = grid_inv(a, grid.qmax), s = grid_scale(a, grid.qmax);
    if (lane == 0 && scales) scales[gi] = s;
    for (int64_t i = lane; i < g; i += kWave) {
      const float z = load1(src + i);
      const float q = grid_code(z, inv, grid);
      codes[r * cols + c0 + i] = int8_t(int(q));
      const float e = __fmul_rn(q, s) - z;
      err += e * e;
    }
  }
  if (partial) block_store_partial(err, partial);
}

// One thread per (group, column), any group length.
template <typename Tag>
__global__ __launch_bounds__(256) void rtn_row_any(
    const typename Tag::elem* __restrict__ W, int64_t rows, int64_t cols, int64_t ld, int64_t g,
    QGrid grid, int8_t* __restrict__ codes, float* __restrict__ scales, double* __restrict__ partial) {
  const int64_t total = (rows / g) * cols;
  float err = 0.f;
  for (int64_t id = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; id < total;
       id += int64_t(gridDim.x) * blockDim.x) {
    const int64_t gr = id / cols, c = id - gr * cols;
    const typename Tag::elem* src = W + gr * g * ld + c;
    float a = 0.f;
    for (int64_t i = 0; i < g; ++i) a = fmaxf(a, fabsf(load1(src + i * ld)));
    const float inv = grid_inv(a, grid.qmax), s = grid_scale(a, grid.qmax);
    if (scales) scales[id] = s;
    for (int64_t i = 0; i < g; ++i) {
      const float z = load1(src + i * ld);
      const float q = grid_code(z, inv, grid);
      codes[(gr * g + i) * cols + c] = int8_t(int(q));
      const float e = __fmul_rn(q, s) - z;
      err += e * e;
    }
  }
  if (partial) block_store_partial(err, partial);
}

// ---- the min/max grid of the paper's Eq. (1) ------------------------------------------------
// Single-precision recipe: r = fl(max - min), inv = min(fl(levels / r), FLT_MAX) (0 for a
// constant group), q = clamp(rint(fl(fl(z - min) * inv)), 0, levels), s = fl(r / levels),
// dequantized value fl(fl(q * s) + min); levels = 2^b - 1.
struct MinMaxGrid { float levels; };
__device__ __forceinline__ float mm_inv(float r, float levels) {
  return r > 0.f ? fminf(__fdiv_rn(levels, r), FLT_MAX) : 0.f;
}
__device__ __forceinline__ float mm_code(float z, float lo, float inv, float levels) {
  const float q = __builtin_rintf(__fmul_rn(__fsub_rn(z, lo), inv));
  return fminf(fmaxf(q, 0.f), levels);
}

// groups along the contiguous axis, g = 4 * LPG <= 256 (same lane ownership as rtn_col_fast)
template <typename Tag, int LPG, bool DENSE>
__global__ __launch_bounds__(kColThreads) void rtn_col_minmax_fast(
    const typename Tag::elem* __restrict__ W, uint32_t nvec, uint32_t cols4, int64_t ld, float levels,
    uint32_t* __restrict__ codes, float* __restrict__ scales, float* __restrict__ mins,
    double* __restrict__ partial) {
  const uint32_t base = blockIdx.x * (kColThreads * kColUnroll) + threadIdx.x;
  float err = 0.f;
#pragma unroll
  for (int j = 0; j < kColUnroll; ++j) {
    const uint32_t v = base + j * kColThreads;
    const bool live = v < nvec;
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) {
      size_t off;
      if constexpr (DENSE) {
        off = size_t(v) * 4;
      } else {
        const uint32_t r = v / cols4;
        off = size_t(r) * ld + size_t(v - r * cols4) * 4;
      }
      x = load4(W + off);
    }
    float hi = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
    float nlo = fmaxf(fmaxf(-x.x, -x.y), fmaxf(-x.z, -x.w));     // -min, so that one reduction serves both
    hi = cluster_allmax<LPG>(hi);
    nlo = cluster_allmax<LPG>(nlo);
    const float lo = -nlo, r = __fsub_rn(hi, lo);
    const float inv = mm_inv(r, levels), s = __fdiv_rn(r, levels);
    const float q0 = mm_code(x.x, lo, inv, levels), q1 = mm_code(x.y, lo, inv, levels);
    const float q2 = mm_code(x.z, lo, inv, levels), q3 = mm_code(x.w, lo, inv, levels);
    if (live) {
      codes[v] = uint32_t(q0) | (uint32_t(q1) << 8) | (uint32_t(q2) << 16) | (uint32_t(q3) << 24);
      if ((threadIdx.x % LPG) == 0) {
        if (scales) scales[v / LPG] = s;
        if (mins) mins[v / LPG] = lo;
      }
      if (partial) {
        const float e0 = __fadd_rn(__fmul_rn(q0, s), lo) - x.x, e1 = __fadd_rn(__fmul_rn(q1, s), lo) - x.y;
        const float e2 = __fadd_rn(__fmul_rn(q2, s), lo) - x.z, e3 = __fadd_rn(__fmul_rn(q3, s), lo) - x.w;
        err += e0 * e0 + e1 * e1 + e2 * e2 + e3 * e3;
      }
    }
  }
  if (partial) block_store_partial(err, partial);
}

// One wave per group along the contiguous axis, group length a multiple of 4 (whole channels
// included): 128-bit loads, four codes per 32-bit store; the second pass re-reads the group
// from cache.
template <typename Tag>
__global__ __launch_bounds__(256) void rtn_col_minmax_vec(
    const typename Tag::elem* __restrict__ W, int64_t rows, int64_t cols, int64_t ld, int64_t g, float levels,
    uint8_t* __restrict__ codes, float* __restrict__ scales, float* __restrict__ mins,
    double* __restrict__ partial) {
  const int lane = threadIdx.x % kWave;
  const int64_t gpr = cols / g, ngroups = rows * gpr;
  const int64_t wave0 = int64_t(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t wstride = int64_t(gridDim.x) * (blockDim.x / kWave);
  float err = 0.f;
  for (int64_t gi = wave0; gi < ngroups; gi += wstride) {
    const int64_t r = gi / gpr, c0 = (gi - r * gpr) * g;
    const typename Tag::elem* src = W + r * ld + c0;
    float hi = -FLT_MAX, nlo = -FLT_MAX;
    for (int64_t i = int64_t(lane) * 4; i < g; i += kWave * 4) {
      const float4 z = load4(src + i);
      hi = fmaxf(hi, fmaxf(fmaxf(z.x, z.y), fmaxf(z.z, z.w)));
      nlo = fmaxf(nlo, fmaxf(fmaxf(-z.x, -z.y), fmaxf(-z.z, -z.w)));
    }
    hi = cluster_allmax<64>(hi);
    nlo = cluster_allmax<64>(nlo);
    const float lo = -nlo, rg = __fsub_rn(hi, lo);
    const float inv = mm_inv(rg, levels), s = __fdiv_rn(rg, levels);
    if (lane == 0) {
      if (scales) scales[gi] = s;
      if (mins) mins[gi] = lo;
    }
    for (int64_t i = int64_t(lane) * 4; i < g; i += kWave * 4) {
      const float4 z = load4(src + i);
      const float q0 = mm_code(z.x, lo, inv, levels), q1 = mm_code(z.y, lo, inv, levels);
      const float q2 = mm_code(z.z, lo, inv, levels), q3 = mm_code(z.w, lo, inv, levels);
      *reinterpret_cast<uint32_t*>(codes + r * cols + c0 + i) =
          uint32_t(q0) | (uint32_t(q1) << 8) | (uint32_t(q2) << 16) | (uint32_t(q3) << 24);
      if (partial) {
        const float e0 = __fadd_rn(__fmul_rn(q0, s), lo) - z.x, e1 = __fadd_rn(__fmul_rn(q1, s), lo) - z.y;
        const float e2 = __fadd_rn(__fmul_rn(q2, s), lo) - z.z, e3 = __fadd_rn(__fmul_rn(q3, s), lo) - z.w;
        err += e0 * e0 + e1 * e1 + e2 * e2 + e3 * e3;
      }
    }
  }
  if (partial) block_store_partial(err, partial);
}

// One wave per group along the contiguous axis, any group length.
template <typename Tag>
__global__ __launch_bounds__(256) void rtn_col_minmax_any(
    const typename Tag::elem* __restrict__ W, int64_t rows, int64_t cols, int64_t ld, int64_t g, float levels,
    uint8_t* __restrict__ codes, float* __restrict__ scales, float* __restrict__ mins,
    double* __restrict__ partial) {
  const int lane = threadIdx.x % kWave;
  const int64_t gpr = cols / g, ngroups = rows * gpr;
  const int64_t wave0 = int64_t(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t wstride = int64_t(gridDim.x) * (blockDim.x / kWave);
  float err = 0.f;
  for (int64_t gi = wave0; gi < ngroups; gi += wstride) {
    const int64_t r = gi / gpr, c0 = (gi - r * gpr) * g;
    const typename Tag::elem* src = W + r * ld + c0;
    float hi = -FLT_MAX, nlo = -FLT_MAX;
    for (int64_t i = lane; i < g; i += kWave) {
      const float z = load1(src + i);
      hi = fmaxf(hi, z);
      nlo = fmaxf(nlo, -z);
    }
    hi = cluster_allmax<64>(hi);
    nlo = cluster_allmax<64>(nlo);
    const float lo = -nlo, rg = __fsub_rn(hi, lo);
    const float inv = mm_inv(rg, levels), s = __fdiv_rn(rg, levels);
    if (lane == 0) {
      if (scales) scales[gi] = s;
      if (mins) mins[gi] = lo;
    }
    for (int64_t i = lane; i < g; i += kWave) {
      const float z = load1(src + i);
      const float q = mm_code(z, lo, inv, levels);
      codes[r * cols + c0 + i] = uint8_t(int(q));
      const float e = __fadd_rn(__fmul_rn(q, s), lo) - z;
      err += e * e;
    }
  }
  if (partial) block_store_partial(err, partial);
}

// One thread per (group, column): groups along the strided axis, any group length.
template <typename Tag>
__global__ __launch_bounds__(256) void rtn_row_minmax_any(
    const typename Tag::elem* __restrict__ W, int64_t rows, int64_t cols, int64_t ld, int64_t g, float levels,
    uint8_t* __restrict__ codes, float* __restrict__ scales, float* __restrict__ mins,
    double* __restrict__ partial) {
  const int64_t total = (rows / g) * cols;
  float err = 0.f;
  for (int64_t id = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; id < total;
       id += int64_t(gridDim.x) * blockDim.x) {
    const int64_t gr = id / cols, c = id - gr * cols;
    const typename Tag::elem* src = W + gr * g * ld + c;
    float hi = -FLT_MAX, lo = FLT_MAX;
    for (int64_t i = 0; i < g; ++i) {
      const float z = load1(src + i * ld);
      hi = fmaxf(hi, z);
      lo = fminf(lo, z);
    }
    const float rg = __fsub_rn(hi, lo);
    const float inv = mm_inv(rg, levels), s = __fdiv_rn(rg, levels);
    if (scales) scales[id] = s;
    if (mins) mins[id] = lo;
    for (int64_t i = 0; i < g; ++i) {
      const float z = load1(src + i * ld);
      const float q = mm_code(z, lo, inv, levels);
      codes[(gr * g + i) * cols + c] = uint8_t(int(q));
      const float e = __fadd_rn(__fmul_rn(q, s), lo) - z;
      err += e * e;
    }
  }
  if (partial) block_store_partial(err, partial);
}

__global__ __launch_bounds__(256) void sum_partials_kernel(const double* __restrict__ partial, int n,
                                                            float* __restrict__ out) {
  __shared__ double red[256];
  double t = 0;
  for (int i = threadIdx.x; i < n; i += 256) t += partial[i];
  red[threadIdx.x] = t;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = float(red[0]);
}

template <typename Tag, int LPG>
void launch_col_fast(const RtnArgs& a, uint32_t nblk, hipStream_t st) {
  using E = typename Tag::elem;
  const uint32_t nvec = uint32_t(a.rows * a.cols / 4), cols4 = uint32_t(a.cols / 4);
  if (a.ld == a.cols)
    hipLaunchKernelGGL((rtn_col_fast<Tag, LPG, true>), dim3(nblk), dim3(kColThreads), 0, st,
                       (const E*)a.W, nvec, cols4, a.ld, a.grid, (uint32_t*)a.codes, a.scales, a.partial);
  else
    hipLaunchKernelGGL((rtn_col_fast<Tag, LPG, false>), dim3(nblk), dim3(kColThreads), 0, st,
                       (const E*)a.W, nvec, cols4, a.ld, a.grid, (uint32_t*)a.codes, a.scales, a.partial);
}

template <typename Tag>
int launch_rtn_typed(const RtnArgs& a, hipStream_t st, int* nparts) {
  using E = typename Tag::elem;
  const int64_t line = a.axis == CAFEQ_AXIS_COL ? a.cols : a.rows;
  const int64_t g = a.group == 0 ? line : a.group;
  *nparts = 0;
  if (a.axis == CAFEQ_AXIS_COL) {
    const bool pow2 = (g & (g - 1)) == 0;
    if (pow2 && g >= 4 && g <= 256 && a.rows * a.cols / 4 < (int64_t(1) << 31)) {
      const int64_t nvec = a.rows * a.cols / 4;
      const uint32_t nblk = uint32_t((nvec + kColThreads * kColUnroll - 1) / (kColThreads * kColUnroll));
      *nparts = int(nblk);
      switch (g / 4) {
        case 1: launch_col_fast<Tag, 1>(a, nblk, st); break;
        case 2: launch_col_fast<Tag, 2>(a, nblk, st); break;
        case 4: launch_col_fast<Tag, 4>(a, nblk, st); break;
        case 8: launch_col_fast<Tag, 8>(a, nblk, st); break;
        case 16: launch_col_fast<Tag, 16>(a, nblk, st); break;
        case 32: launch_col_fast<Tag, 32>(a, nblk, st); break;
        default: launch_col_fast<Tag, 64>(a, nblk, st); break;
      }
    } else {
      const int64_t ngroups = a.rows * (a.cols / g);
      const int nblk = int(std::min<int64_t>((ngroups + 3) / 4, 4096));
      *nparts = nblk;
      if (g % 4 == 0 && a.ld % 4 == 0 && a.cols % 4 == 0)
        hipLaunchKernelGGL((rtn_col_vec<Tag>), dim3(nblk), dim3(256), 0, st, (const E*)a.W, a.rows, a.cols,
                           a.ld, g, a.grid, a.codes, a.scales, a.partial);
      else
        hipLaunchKernelGGL((rtn_col_any<Tag>), dim3(nblk), dim3(256), 0, st, (const E*)a.W, a.rows, a.cols,
                           a.ld, g, a.grid, a.codes, a.scales, a.partial);
    }
  } else {
    const int nw = int(g / kRowRPW);
    if (g % kRowRPW == 0 && (nw == 1 || nw == 2 || nw == 4 || nw == 8 || nw == 16) &&
        a.rows / g < 65536) {
      dim3 grid(unsigned((a.cols + 255) / 256), unsigned(a.rows / g));
      *nparts = int(grid.x * grid.y);
#define CAFEQ_ROW_CASE(NW)                                                                          \
  case NW:                                                                                          \
    hipLaunchKernelGGL((rtn_row_fast<Tag, NW>), grid, dim3(NW* kWave), 0, st, (const E*)a.W, a.cols, \
                       a.ld, a.grid, a.codes, a.scales, a.partial);                                 \
    break;
      switch (nw) {
        CAFEQ_ROW_CASE(1)
        CAFEQ_ROW_CASE(2)
        CAFEQ_ROW_CASE(4)
        CAFEQ_ROW_CASE(8)
        CAFEQ_ROW_CASE(16)
      }
#undef CAFEQ_ROW_CASE
    } else {
      const int64_t total = (a.rows / g) * a.cols;
      const int nblk = int(std::min<int64_t>((total + 255) / 256, 4096));
      *nparts = nblk;
      hipLaunchKernelGGL((rtn_row_any<Tag>), dim3(nblk), dim3(256), 0, st, (const E*)a.W, a.rows, a.cols,
                         a.ld, g, a.grid, a.codes, a.scales, a.partial);
    }
  }
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

template <typename Tag, int LPG>
void launch_col_minmax_fast(const RtnArgs& a, float levels, uint32_t nblk, hipStream_t st) {
  using E = typename Tag::elem;
  const uint32_t nvec = uint32_t(a.rows * a.cols / 4), cols4 = uint32_t(a.cols / 4);
  if (a.ld == a.cols)
    hipLaunchKernelGGL((rtn_col_minmax_fast<Tag, LPG, true>), dim3(nblk), dim3(kColThreads), 0, st, (const E*)a.W,
                       nvec, cols4, a.ld, levels, (uint32_t*)a.codes, a.scales, a.mins, a.partial);
  else
    hipLaunchKernelGGL((rtn_col_minmax_fast<Tag, LPG, false>), dim3(nblk), dim3(kColThreads), 0, st, (const E*)a.W,
                       nvec, cols4, a.ld, levels, (uint32_t*)a.codes, a.scales, a.mins, a.partial);
}

template <typename Tag>
int launch_minmax_typed(const RtnArgs& a, float levels, hipStream_t st, int* nparts) {
  using E = typename Tag::elem;
  const int64_t line = a.axis == CAFEQ_AXIS_COL ? a.cols : a.rows;
  const int64_t g = a.group == 0 ? line : a.group;
  if (a.axis == CAFEQ_AXIS_COL) {
    const bool pow2 = (g & (g - 1)) == 0;
    if (pow2 && g >= 4 && g <= 256 && a.rows * a.cols / 4 < (int64_t(1) << 31)) {
      const int64_t nvec = a.rows * a.cols / 4;
      const uint32_t nblk = uint32_t((nvec + kColThreads * kColUnroll - 1) / (kColThreads * kColUnroll));
      *nparts = int(nblk);
      switch (g / 4) {
        case 1: launch_col_minmax_fast<Tag, 1>(a, levels, nblk, st); break;
        case 2: launch_col_minmax_fast<Tag, 2>(a, levels, nblk, st); break;
        case 4: launch_col_minmax_fast<Tag, 4>(a, levels, nblk, st); break;
        case 8: launch_col_minmax_fast<Tag, 8>(a, levels, nblk, st); break;
        case 16: launch_col_minmax_fast<Tag, 16>(a, levels, nblk, st); break;
        case 32: launch_col_minmax_fast<Tag, 32>(a, levels, nblk, st); break;
        default: launch_col_minmax_fast<Tag, 64>(a, levels, nblk, st); break;
      }
    } else {
      const int64_t ngroups = a.rows * (a.cols / g);
      const int nblk = int(std::min<int64_t>((ngroups + 3) / 4, 4096));
      *nparts = nblk;
      // load4 needs 16-byte (float32) / 8-byte (bfloat16) aligned groups; the code stores 4-byte aligned ones
      if (g % 4 == 0 && a.ld % 4 == 0 && a.cols % 4 == 0)
        hipLaunchKernelGGL((rtn_col_minmax_vec<Tag>), dim3(nblk), dim3(256), 0, st, (const E*)a.W, a.rows, a.cols,
                           a.ld, g, levels, (uint8_t*)a.codes, a.scales, a.mins, a.partial);
      else
        hipLaunchKernelGGL((rtn_col_minmax_any<Tag>), dim3(nblk), dim3(256), 0, st, (const E*)a.W, a.rows, a.cols,
                           a.ld, g, levels, (uint8_t*)a.codes, a.scales, a.mins, a.partial);
    }
  } else {
    const int64_t total = (a.rows / g) * a.cols;
    const int nblk = int(std::min<int64_t>((total + 255) / 256, 4096));
    *nparts = nblk;
    hipLaunchKernelGGL((rtn_row_minmax_any<Tag>), dim3(nblk), dim3(256), 0, st, (const E*)a.W, a.rows, a.cols,
                       a.ld, g, levels, (uint8_t*)a.codes, a.scales, a.mins, a.partial);
  }
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // namespace

int launch_rtn_minmax(const RtnArgs& a, int bits, hipStream_t st) {
  int nparts = 0;
  const float levels = float((1 << bits) - 1);
  int rc = a.dtype == CAFEQ_BF16 ? launch_minmax_typed<BF16Tag>(a, levels, st, &nparts)
                                 : launch_minmax_typed<F32Tag>(a, levels, st, &nparts);
  if (rc != CAFEQ_OK) return rc;
  if (a.partial) {
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, a.partial, nparts, a.err_sq);
    CAFEQ_CHECK_LAUNCH();
  }
  return CAFEQ_OK;
}

size_t rtn_partials_capacity(int64_t rows, int64_t cols) {
  // upper bound on the number of workgroups any of the four kernels launches
  const int64_t fast = (rows * cols / 4 + kColThreads * kColUnroll - 1) / (kColThreads * kColUnroll);
  const int64_t rowfast = ((cols + 255) / 256) * ((rows + 15) / 16);
  return size_t(std::max<int64_t>(std::max(fast, rowfast), 4096));
}

int launch_rtn(const RtnArgs& a, hipStream_t st) {
  int nparts = 0;
  int rc = a.dtype == CAFEQ_BF16 ? launch_rtn_typed<BF16Tag>(a, st, &nparts)
                                 : launch_rtn_typed<F32Tag>(a, st, &nparts);
  if (rc != CAFEQ_OK) return rc;
  if (a.partial) {
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, a.partial, nparts, a.err_sq);
    CAFEQ_CHECK_LAUNCH();
  }
  return CAFEQ_OK;
}

}  // namespace cafeq
