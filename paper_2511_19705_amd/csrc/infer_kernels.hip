// Inference side of a single transformed matrix (paper Sec. 4.1, the display Y^ = X M^-1 Q(MW)):
// the activations take the blockwise inverse transform, then the product with the dequantized
// transformed weight.  With this library's [out][in] weights and Z = W . blockdiag(T):
//   x'[b*k + i] = sum_j Tinv[b][i][j] x[b*k + j]          (act_transform_kernel, d*k multiply-adds)
//   y[o]        = sum_c s[o][c / g] q[o][c] x'[c]          (dequant_gemv_kernel, one byte per weight)
// The second kernel is the layer itself in the few-token (matrix-vector) regime and is bound by
// reading the codes once from HBM; the first is the extra work the transform adds, the quantity
// the paper's block-size table reports as extra FLOPs / extra wall-clock time.
#include "cafeq_common.hpp"
#include "cafeq_internal.hpp"

namespace cafeq {
namespace {

constexpr int kTokA = 4;    // tokens per workgroup of the activation transform
constexpr int kRowsA = 16;  // rows of Tinv per wave

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }

// The inverse blocks are one long list of d rows of K contiguous floats (row R of block R / K).  A wave
// owns kRowsA consecutive rows: each 128-bit load instruction covers 256 / K rows (K / 4 lanes per row),
// every lane multiplies its four weights with the matching four activations (held in registers), and
// the per-row sums are formed by a butterfly that halves the list of values while it doubles the span
// of lanes (so kRowsA rows cost about kRowsA exchanges, not 6 each).  No LDS, no barriers.
template <int K>
__global__ __launch_bounds__(256) void act_transform_kernel(const float* __restrict__ X, int64_t ldx, int n,
                                                            const float* __restrict__ Tinv, float* __restrict__ Xp,
                                                            int64_t ldp, int64_t d) {
  constexpr int LPR = K / 4;           // lanes per row
  constexpr int RPL = 64 / LPR;        // rows per load instruction
  constexpr int NL = kRowsA / RPL;     // load instructions per wave
  constexpr int TS = ilog2(NL);        // halving steps
  static_assert(LPR <= 64 && (1 << TS) <= LPR, "block size");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row0 = (int64_t(blockIdx.x) * 4 + wave) * kRowsA;
  if (row0 >= d) return;
  const int t0 = blockIdx.y * kTokA, nt = min(kTokA, n - t0);
  const int sub = lane / LPR, cl = lane % LPR;
  const int64_t col0 = row0 / K * K + cl * 4;
  float4 xv[kTokA];
#pragma unroll
  for (int t = 0; t < kTokA; ++t)
    xv[t] = t < nt ? *reinterpret_cast<const float4*>(X + int64_t(t0 + t) * ldx + col0) : make_float4(0.f, 0.f, 0.f, 0.f);
  float4 p[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i)
    p[i] = *reinterpret_cast<const float4*>(Tinv + (row0 + i * RPL + sub) * K + cl * 4);
  int idx = 0;   // which of the NL values this lane ends up with
#pragma unroll
  for (int s = 0; s < TS; ++s) idx += ((lane >> s) & 1) * (NL >> (s + 1));
#pragma unroll
  for (int t = 0; t < kTokA; ++t) {
    if (t >= nt) break;
    float v[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i)
      v[i] = fmaf(p[i].x, xv[t].x, fmaf(p[i].y, xv[t].y, fmaf(p[i].z, xv[t].z, p[i].w * xv[t].w)));
#pragma unroll
    for (int s = 0; s < TS; ++s) {
      const int half = NL >> (s + 1);
      // bitwise selects (a mask per lane) keep the list in registers with constant indices
      const uint32_t um = 0u - uint32_t((lane >> s) & 1);
#pragma unroll
      for (int j = 0; j < half; ++j) {
        const uint32_t lo = __float_as_uint(v[j]), hi = __float_as_uint(v[j + half]);
        const float keep = __uint_as_float((lo & ~um) | (hi & um));
        const float send = __uint_as_float((hi & ~um) | (lo & um));
        v[j] = keep + __shfl_xor(send, 1 << s);
      }
    }
#pragma unroll
    for (int m = 1 << TS; m < LPR; m <<= 1) v[0] += __shfl_xor(v[0], m);
    if ((cl >> TS) == 0) Xp[int64_t(t0 + t) * ldp + row0 + idx * RPL + sub] = v[0];
  }
}

struct GemvArgs {
  const int8_t* codes;   // [out][in]
  const float* scales;   // [out][in / g]
  const float* xp;       // [NT][in] (leading dimension ldp)
  float* y;              // [NT][ldy]
  int64_t out, in, ldp, ldy;
  int g, ngrp;           // group length (elements), groups per row
  int rows_per_wg;
};

constexpr int kRowsMax = 4;  // most rows in flight per workgroup; rows per workgroup are a multiple of it
// rows in flight: fewer when the activations already fill the register file
constexpr int rows_in_flight(int nt, int ch) { return nt * ch <= 3 ? 4 : (nt * ch <= 6 ? 2 : 1); }

// signed byte `i` of a dword as a float (byte-select conversion)
template <int I>
__device__ __forceinline__ float byte_f(uint32_t w) {
  return float(int(int8_t(w >> (8 * I))));
}

// Every thread keeps, for CH chunks of 16 consecutive inputs, the NT tokens' transformed
// activations in registers; the workgroup then streams its rows of codes (one 128-bit load per
// thread, chunk and row: each wave reads 1 KB contiguous), multiplies, and reduces over the
// threads once per batch of rows.
template <int NT, int CH>
__global__ __launch_bounds__(512) void dequant_gemv_kernel(const GemvArgs a) {
  constexpr int kRowsB = rows_in_flight(NT, CH);
  __shared__ float red[8][kRowsB * NT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthr = blockDim.x, nwave = nthr >> 6;
  const int nchunk = int(a.in >> 4);
  float x[NT][CH][16];
  bool live[CH];
  int gi[CH];   // the chunk's quantization group
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = tid + i * nthr;
    live[i] = c < nchunk;
    gi[i] = (c * 16) / a.g;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const float* src = a.xp + int64_t(t) * a.ldp + int64_t(c) * 16;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = live[i] ? *reinterpret_cast<const float4*>(src + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
        x[t][i][4 * q] = v.x; x[t][i][4 * q + 1] = v.y; x[t][i][4 * q + 2] = v.z; x[t][i][4 * q + 3] = v.w;
      }
    }
  }
  const int64_t r_begin = int64_t(blockIdx.x) * a.rows_per_wg;
  const int64_t r_end = min(a.out, r_begin + a.rows_per_wg);
  for (int64_t r0 = r_begin; r0 < r_end; r0 += kRowsB) {
    uint4 cw[kRowsB][CH];
    float sc[kRowsB][CH];
#pragma unroll
    for (int r = 0; r < kRowsB; ++r) {
      const bool rv = r0 + r < r_end;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const int c = tid + i * nthr;
        const bool v = rv && live[i];
        cw[r][i] = v ? *reinterpret_cast<const uint4*>(a.codes + (r0 + r) * a.in + int64_t(c) * 16)
                     : make_uint4(0u, 0u, 0u, 0u);
        sc[r][i] = v ? a.scales[(r0 + r) * a.ngrp + gi[i]] : 0.f;
      }
    }
    float acc[kRowsB][NT];
#pragma unroll
    for (int r = 0; r < kRowsB; ++r) {
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[r][t] = 0.f;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const uint32_t w[4] = {cw[r][i].x, cw[r][i].y, cw[r][i].z, cw[r][i].w};
        float q[16];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          q[4 * d] = byte_f<0>(w[d]); q[4 * d + 1] = byte_f<1>(w[d]);
          q[4 * d + 2] = byte_f<2>(w[d]); q[4 * d + 3] = byte_f<3>(w[d]);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float d0 = 0.f, d1 = 0.f;   // two chains per chunk
#pragma unroll
          for (int e = 0; e < 16; e += 2) {
            d0 = fmaf(q[e], x[t][i][e], d0);
            d1 = fmaf(q[e + 1], x[t][i][e + 1], d1);
          }
          acc[r][t] = fmaf(sc[r][i], d0 + d1, acc[r][t]);
        }
      }
    }
    // over the threads: inside each wave, then across the waves through LDS
#pragma unroll
    for (int r = 0; r < kRowsB; ++r)
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const float v = wave_sum(acc[r][t]);
        if (lane == 0) red[wave][r * NT + t] = v;
      }
    __syncthreads();
    if (tid < kRowsB * NT) {
      float v = 0.f;
      for (int w = 0; w < nwave; ++w) v += red[w][tid];
      const int r = tid / NT, t = tid - r * NT;
      if (r0 + r < r_end) a.y[int64_t(t) * a.ldy + r0 + r] = v;
    }
    __syncthreads();
  }
}

// chunks of 16 inputs spread over T threads x CH chunks each: the pair with the fewest idle slots
bool pick_shape(int64_t in, int ch_max, int* T, int* CH) {
  const int64_t chunks = in / 16;
  int64_t best = -1;
  for (int ch = 1; ch <= ch_max; ++ch) {
    const int64_t per = (chunks + ch - 1) / ch;
    const int64_t t = (per + 63) / 64 * 64;
    if (t > 512) continue;
    const int64_t slots = t * ch;
    if (best < 0 || slots < best) { best = slots; *T = int(t); *CH = ch; }
  }
  return best >= 0;
}

template <int NT>
int launch_gemv_nt(const GemvArgs& a, int T, int CH, unsigned nwg, hipStream_t st) {
#define CAFEQ_GEMV(C) case C: hipLaunchKernelGGL((dequant_gemv_kernel<NT, C>), dim3(nwg), dim3(T), 0, st, a); break
  switch (CH) {
    CAFEQ_GEMV(1); CAFEQ_GEMV(2);
    case 3: if constexpr (NT <= 2) { hipLaunchKernelGGL((dequant_gemv_kernel<NT, 3>), dim3(nwg), dim3(T), 0, st, a); break; } else return CAFEQ_ERR_UNSUPPORTED;
    case 4: if constexpr (NT <= 2) { hipLaunchKernelGGL((dequant_gemv_kernel<NT, 4>), dim3(nwg), dim3(T), 0, st, a); break; } else return CAFEQ_ERR_UNSUPPORTED;
    case 5: if constexpr (NT == 1) { hipLaunchKernelGGL((dequant_gemv_kernel<NT, 5>), dim3(nwg), dim3(T), 0, st, a); break; } else return CAFEQ_ERR_UNSUPPORTED;
    case 6: if constexpr (NT == 1) { hipLaunchKernelGGL((dequant_gemv_kernel<NT, 6>), dim3(nwg), dim3(T), 0, st, a); break; } else return CAFEQ_ERR_UNSUPPORTED;
    case 7: if constexpr (NT == 1) { hipLaunchKernelGGL((dequant_gemv_kernel<NT, 7>), dim3(nwg), dim3(T), 0, st, a); break; } else return CAFEQ_ERR_UNSUPPORTED;
    case 8: if constexpr (NT == 1) { hipLaunchKernelGGL((dequant_gemv_kernel<NT, 8>), dim3(nwg), dim3(T), 0, st, a); break; } else return CAFEQ_ERR_UNSUPPORTED;
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
#undef CAFEQ_GEMV
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // namespace
}  // namespace cafeq

using namespace cafeq;

extern "C" {

size_t cafeq_infer_workspace_bytes(int n, int64_t in) {
  if (n < 1 || in < 1) return 0;
  return align_up(size_t(n) * size_t(in) * sizeof(float), 256);
}

int cafeq_infer_single(const float* X, int n, int64_t ldx, const cafeq_xform* xf, const int8_t* codes,
                       const float* scales, int64_t out, int64_t in, int group, float* Y, int64_t ldy, void* ws,
                       void* stream) {
  if (!X || !codes || !scales || !Y) return CAFEQ_ERR_INVALID_ARG;
  if (n < 1 || out < 1 || in < 16 || ldx < in || ldy < out) return CAFEQ_ERR_BAD_SHAPE;
  const int64_t g = group == 0 ? in : group;
  if (in % 16 != 0 || g < 16 || g % 16 != 0 || in % g != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (in > 65536 || in / g > INT32_MAX) return CAFEQ_ERR_UNSUPPORTED;
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (!al16(X) || !al16(codes) || ldx % 4 != 0) return CAFEQ_ERR_BAD_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const float* xp = X;
  int64_t ldp = ldx;
  if (xf) {
    if (!xf->Tinv) return CAFEQ_ERR_INVALID_ARG;
    if (xf->rep != 1 || int64_t(xf->nb) * xf->k != in) return CAFEQ_ERR_BAD_SHAPE;
    if (!al16(xf->Tinv)) return CAFEQ_ERR_BAD_ALIGN;
    if (!ws) return CAFEQ_ERR_WORKSPACE;
    if (!al16(ws)) return CAFEQ_ERR_BAD_ALIGN;
    float* dst = static_cast<float*>(ws);
    const dim3 grid(unsigned((in + 4 * kRowsA - 1) / (4 * kRowsA)), unsigned((n + kTokA - 1) / kTokA));
    switch (xf->k) {
      case 32: hipLaunchKernelGGL(act_transform_kernel<32>, grid, dim3(256), 0, st, X, ldx, n, xf->Tinv, dst, in, in); break;
      case 64: hipLaunchKernelGGL(act_transform_kernel<64>, grid, dim3(256), 0, st, X, ldx, n, xf->Tinv, dst, in, in); break;
      case 128: hipLaunchKernelGGL(act_transform_kernel<128>, grid, dim3(256), 0, st, X, ldx, n, xf->Tinv, dst, in, in); break;
      case 256: hipLaunchKernelGGL(act_transform_kernel<256>, grid, dim3(256), 0, st, X, ldx, n, xf->Tinv, dst, in, in); break;
      default: return CAFEQ_ERR_UNSUPPORTED;
    }
    CAFEQ_CHECK_LAUNCH();
    xp = dst;
    ldp = in;
  }
  GemvArgs a;
  a.codes = codes; a.scales = scales; a.out = out; a.in = in; a.ldy = ldy; a.ldp = ldp;
  a.g = int(g); a.ngrp = int(in / g);
  // about two workgroups per compute unit, whole batches of rows each
  int64_t rpw = (out + 511) / 512;
  rpw = (rpw + kRowsMax - 1) / kRowsMax * kRowsMax;
  a.rows_per_wg = int(rpw);
  const unsigned nwg = unsigned((out + rpw - 1) / rpw);
  for (int t0 = 0; t0 < n;) {
    const int left = n - t0;
    int T = 0, CH = 0, nt = 0;
    if (left >= 4 && pick_shape(in, 2, &T, &CH)) nt = 4;
    else if (left >= 2 && pick_shape(in, 4, &T, &CH)) nt = 2;
    else if (pick_shape(in, 8, &T, &CH)) nt = 1;
    else return CAFEQ_ERR_UNSUPPORTED;
    a.xp = xp + int64_t(t0) * ldp;
    a.y = Y + int64_t(t0) * ldy;
    const int rc = nt == 4 ? launch_gemv_nt<4>(a, T, CH, nwg, st)
                 : nt == 2 ? launch_gemv_nt<2>(a, T, CH, nwg, st)
                           : launch_gemv_nt<1>(a, T, CH, nwg, st);
    if (rc) return rc;
    t0 += nt;
  }
  return CAFEQ_OK;
}

}  // extern "C"
