// Device-side helpers shared by the gfx950 kernels of the CafeQ hot-path library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <float.h>

#include "cafeq.h"

namespace cafeq {

constexpr int kWave = 64;

// ---------------------------------------------------------------------------
// storage types
// ---------------------------------------------------------------------------
struct F32Tag { using elem = float; static constexpr int dtype = CAFEQ_F32; };
struct BF16Tag { using elem = uint16_t; static constexpr int dtype = CAFEQ_BF16; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Four consecutive elements starting at p (16-byte aligned for float, 8-byte for bf16).
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const uint16_t* p) {
  uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u),
                     __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u));
}
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// ---------------------------------------------------------------------------
// cross-lane data movement (wave64)
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// max over aligned clusters of LANES consecutive lanes, result in every lane of the cluster.
// quad_perm / row-mirror DPP inside a 16-lane row, LDS-crossbar shuffles across rows.
template <int LANES>
__device__ __forceinline__ float cluster_allmax(float v) {
  if constexpr (LANES >= 2) v = fmaxf(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
  if constexpr (LANES >= 4) v = fmaxf(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
  if constexpr (LANES >= 8) v = fmaxf(v, dpp_mov<0x141>(v));   // row_half_mirror
  if constexpr (LANES >= 16) v = fmaxf(v, dpp_mov<0x140>(v));  // row_mirror
  if constexpr (LANES >= 32) v = fmaxf(v, __shfl_xor(v, 16));
  if constexpr (LANES >= 64) v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  v += dpp_mov<0x140>(v);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
  return v;
}

// ---------------------------------------------------------------------------
// the symmetric absmax grid (single-precision recipe stated in cafeq.h)
// ---------------------------------------------------------------------------
struct QGrid {
  float qmax, qmin;
};
__host__ __device__ inline QGrid make_grid(int bits) {
  QGrid g;
  g.qmax = float((1 << (bits - 1)) - 1);
  g.qmin = -float(1 << (bits - 1));
  return g;
}
// inv = fl(qmax / a) (0 for an all-zero group; capped so a denormal absmax cannot give inf)
__device__ __forceinline__ float grid_inv(float a, float qmax) {
  return a > 0.f ? fminf(__fdiv_rn(qmax, a), FLT_MAX) : 0.f;
}
__device__ __forceinline__ float grid_scale(float a, float qmax) { return __fdiv_rn(a, qmax); }
// code as a float holding an integer in [qmin, qmax]
__device__ __forceinline__ float grid_code(float z, float inv, QGrid g) {
  float r = __builtin_rintf(__fmul_rn(z, inv));
  return fminf(fmaxf(r, g.qmin), g.qmax);
}
__device__ __forceinline__ uint32_t pack4(float q0, float q1, float q2, float q3) {
  return (uint32_t(int(q0)) & 0xFFu) | ((uint32_t(int(q1)) & 0xFFu) << 8) |
         ((uint32_t(int(q2)) & 0xFFu) << 16) | (uint32_t(int(q3)) << 24);
}

// ---------------------------------------------------------------------------
// host-side launch checking
// ---------------------------------------------------------------------------
#define CAFEQ_CHECK_LAUNCH()                                   \
  do {                                                         \
    if (hipGetLastError() != hipSuccess) return CAFEQ_ERR_LAUNCH; \
  } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace cafeq
