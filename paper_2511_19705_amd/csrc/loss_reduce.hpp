// Final reduction of the per-(workgroup, segment) partial headers into the call's losses (fixed-order float64
// sums; for the pair the LogSumExp over all group maxima, paper Sec. 4.2, from per-slot sums of exponentials that
// are relative to per-slot references).  One body, two users: the stand-alone kernel of one workgroup, and the
// gradient pass with one workgroup per block, whose workgroups each repeat it (a few hundred headers from the
// memory-side cache) instead of waiting for a launch of its own; only the workgroup told to writes the results.
// The first 256 threads of the NT-thread workgroup walk the headers -- the summation order does not depend on NT.
#pragma once
#include "xform_core.hpp"

namespace cafeq {

struct LossArgs {
  const float* hdrA; int nslotA;     // member A (or the single matrix)
  const float* hdrB; int nslotB;     // member B (dual only)
  int kind; float beta, t;
  int64_t ngroups;
  float* losses;
  double* lse_ms;                    // out: [m*, S]
};
constexpr int kLossThreads = 256;

// red: 5 * (NT / 64) doubles of LDS.  Returns {m*, S} through m_out / s_out (kLossLse; untouched otherwise).
template <int NT>
__device__ __forceinline__ void reduce_losses_body(const LossArgs& a, double* red, bool write, double* m_out,
                                                   double* s_out) {
  constexpr int NW = NT / 64;
  const bool walker = threadIdx.x < kLossThreads;
  // four sums and one maximum over the workgroup, fixed order
  auto reduce5 = [&](double& v0, double& v1, double& v2, double& v3, double& vmax) {
    for (int k = 1; k < 64; k <<= 1) {
      v0 += __shfl_xor(v0, k); v1 += __shfl_xor(v1, k); v2 += __shfl_xor(v2, k); v3 += __shfl_xor(v3, k);
      vmax = fmax(vmax, __shfl_xor(vmax, k));
    }
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
      red[w] = v0; red[NW + w] = v1; red[2 * NW + w] = v2; red[3 * NW + w] = v3; red[4 * NW + w] = vmax;
    }
    __syncthreads();
    v0 = v1 = v2 = v3 = 0;
    vmax = -INFINITY;
    for (int k = 0; k < NW; ++k) {
      v0 += red[k]; v1 += red[NW + k]; v2 += red[2 * NW + k]; v3 += red[3 * NW + k];
      vmax = fmax(vmax, red[4 * NW + k]);
    }
    __syncthreads();
  };
  if (a.kind == kLossSur) {
    double l2 = 0, ez = 0, ws = 0, su = 0, dummy = -INFINITY;
    if (walker) {
      for (int i = threadIdx.x; i < a.nslotA; i += kLossThreads) {
        const float* h = a.hdrA + size_t(i) * kHdrFloats;
        l2 += h[kHdrL2]; ez += h[kHdrErrZ]; ws += h[kHdrWsq]; su += h[kHdrSur];
      }
    }
    reduce5(l2, ez, ws, su, dummy);
    if (write && threadIdx.x == 0) {
      a.losses[0] = float(l2); a.losses[1] = float(ez); a.losses[2] = float(ws);
      a.losses[3] = float(su * a.beta);
    }
    return;
  }
  // one pass over both members' headers: four sums and the largest reference; each thread keeps
  // its slots' (sum of exponentials, reference) pairs for the second step
  constexpr int kMaxPer = 8;                       // slots per thread held in registers
  const int ntot = a.nslotA + a.nslotB;
  double ezA = 0, ezB = 0, l2A = 0, l2B = 0, m = -INFINITY;
  float sur[kMaxPer], mref[kMaxPer];
  int cnt = 0;
  if (walker) {
    for (int i = threadIdx.x; i < ntot; i += kLossThreads, ++cnt) {
      const bool isA = i < a.nslotA;
      const float* h = isA ? a.hdrA + size_t(i) * kHdrFloats : a.hdrB + size_t(i - a.nslotA) * kHdrFloats;
      const float ez = h[kHdrErrZ], l2 = h[kHdrL2], su = h[kHdrSur], mr = h[kHdrMref];
      if (isA) { ezA += ez; l2A += l2; } else { ezB += ez; l2B += l2; }
      m = fmax(m, double(mr));
      if (cnt < kMaxPer) { sur[cnt] = su; mref[cnt] = mr; }
    }
  }
  reduce5(ezA, ezB, l2A, l2B, m);
  // global normaliser of the exponentials
  double s = 0;
  cnt = 0;
  if (walker) {
    for (int i = threadIdx.x; i < ntot; i += kLossThreads, ++cnt) {
      float su, mr;
      if (cnt < kMaxPer) { su = sur[cnt]; mr = mref[cnt]; }
      else {
        const float* h = i < a.nslotA ? a.hdrA + size_t(i) * kHdrFloats : a.hdrB + size_t(i - a.nslotA) * kHdrFloats;
        su = h[kHdrSur]; mr = h[kHdrMref];
      }
      if (su > 0.f) s += double(su) * exp(double(a.t) * (double(mr) - m));
    }
  }
  double z1 = 0, z2 = 0, z3 = 0, zm = -INFINITY;
  reduce5(s, z1, z2, z3, zm);
  if (write && threadIdx.x == 0) {
    a.losses[0] = float(ezA); a.losses[1] = float(ezB); a.losses[2] = float(l2A); a.losses[3] = float(l2B);
    a.losses[4] = float(m + log(s) / double(a.t));
    a.losses[5] = float(a.ngroups);
    a.lse_ms[0] = m; a.lse_ms[1] = s;
  }
  *m_out = m;
  *s_out = s;
}

}  // namespace cafeq
