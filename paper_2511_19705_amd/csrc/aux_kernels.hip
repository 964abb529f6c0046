// Small kernels around the fused core: squared norms of the inverse transform (the
// (M^-1)_{ij}^2 factors of the paper's surrogate, Sec. 4.1), fixed-order reduction of the
// per-workgroup partials and the k x k products of the gradient's path through M^-1.  All are off the bandwidth path (k x k sized per block).
#include <atomic>
#include "cafeq_internal.hpp"
#include "xform_core.hpp"
#include "loss_reduce.hpp"

namespace cafeq {

namespace {

// rho[b*K + j]: squared norm of row j (by_row) or column j of P_b, summed in float64.  256 / K threads share a
// line (K = 256: one each); they take its elements interleaved and meet in LDS, added in thread order.  A workgroup
// takes nbk consecutive blocks.
// With rG != null the workgroup also writes the sums of rho over groups of G axis indices (what rho_group_kernel
// computes, in its arithmetic: lanes interleaved over a group's indices, then a wave sum):
//   G <= K, G | K, nbk = 1: rG[(b rep + r) (K / G) + q] = sum over indices q G .. q G + G - 1 of block b, for each
//                           of the rep row-blocks that share the block;
//   G = nbk K <= 256, rep = 1: rG[workgroup] = sum over its nbk blocks.
__global__ __launch_bounds__(256) void rho_kernel(const float* __restrict__ P, int K, int by_row,
                                                   float* __restrict__ rho, float* __restrict__ rG, int G, int rep,
                                                   int nbk) {
  __shared__ double part[256];
  __shared__ float line[256];
  const int tpl = 256 / K;                       // threads per line: K is 32, 64, 128 or 256
  // by_row: neighbouring threads share a row (their loads fall into the same cache lines);
  // by column: neighbouring threads take neighbouring columns (coalesced rows)
  const int j = by_row ? threadIdx.x / tpl : threadIdx.x % K;
  const int s = by_row ? threadIdx.x % tpl : threadIdx.x / K;
  for (int bb = 0; bb < nbk; ++bb) {
    const size_t b = size_t(blockIdx.x) * nbk + bb;
    const float* Pb = P + b * K * K;
    double acc = 0;
    for (int i = s; i < K; i += tpl) {
      const float v = by_row ? Pb[j * K + i] : Pb[i * K + j];
      acc += double(v) * v;
    }
    part[s * K + j] = acc;
    __syncthreads();
    if (threadIdx.x < K) {
      double t = part[threadIdx.x];
      for (int q = 1; q < tpl; ++q) t += part[q * K + threadIdx.x];
      rho[b * K + threadIdx.x] = float(t);
      if (rG) line[bb * K + threadIdx.x] = float(t);      // (rG set: nbk K <= 256)
    }
    __syncthreads();
  }
  if (rG == nullptr) return;                     // uniform
  const int lane = threadIdx.x % kWave;
  if (nbk > 1) {
    if (threadIdx.x < kWave) {
      float acc = 0.f;
      for (int e = lane; e < G; e += kWave) acc += line[e];
      acc = wave_sum(acc);
      if (lane == 0) rG[blockIdx.x] = acc;
    }
    return;
  }
  const int ng = K / G;
  for (int q = threadIdx.x / kWave; q < ng; q += 256 / kWave) {
    float acc = 0.f;
    for (int e = lane; e < G; e += kWave) acc += line[q * G + e];
    acc = wave_sum(acc);
    if (lane == 0)
      for (int r = 0; r < rep; ++r) rG[(size_t(blockIdx.x) * rep + r) * ng + q] = acc;
  }
}

// Operand planes of the fused core.  Element [out][in] of the k x k operand -- src_b (trans == 0) or
// src_b^T (trans == 1) -- is split exactly into bfloat16 parts x = hi + mid + lo (+ a residual below
// 2^-24 |x|) and stored in the order the core streams it through its LDS ring:
//   dst[b][stage = in / 32][part][out][32 inputs of the stage]
// with the 32 inputs of a row arranged as four 16-byte chunks (MFMA step c2 = (in % 32) / 16, lane
// half h -> chunk 2*c2 + h, holding inputs 16*c2 + 8u + 4h + e at position 4u + e), the chunk stored
// at chunk ^ ((out >> 2) & 3) (LDS bank swizzle).
struct SplitJob { const float* src; uint16_t* dst; int trans, nplanes; float* fscale; int natural, texp; };   // fscale, texp: see below
struct SplitJobs { SplitJob job[4]; int njobs, K; float* hdr; int64_t nhdr; };   // hdr: partial headers to reset (may be null)
// A job with fscale != null writes TWO float16 planes instead: the block is first scaled by the power of
// two that puts its largest magnitude into [2^texp, 2^(texp+1)) (14: the low parts stay normal numbers; 4: sums of
// 128 products with operands below 2^4 stay below 2^16 -- the matrix cores take denormal float16 inputs exactly), then
// x = hi + lo with both parts rounded to nearest; fscale[b] receives the factor that undoes the scale.
// grid: (nb, njobs): one workgroup per (block, job) walks the K / 32 stages, so that the block's largest
// magnitude (float16 jobs) is found once.
constexpr int kSplitThreads = 1024;
__global__ __launch_bounds__(kSplitThreads) void split_planes_kernel(const SplitJobs js) {
  // a stage's planes are assembled in LDS in their final order and leave as whole 16-byte vectors
  __shared__ __align__(16) uint16_t lds[3 * 256 * 32];
  const int K = js.K, nst = K / 32;
  // partial headers that no workgroup of the core writes (slots nobody owns) must read as empty
  if (js.hdr) {
    const int64_t nthr = int64_t(gridDim.x) * gridDim.y * gridDim.z * kSplitThreads;
    for (int64_t i = ((int64_t(blockIdx.z) * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * kSplitThreads + threadIdx.x;
         i < js.nhdr; i += nthr)
      js.hdr[i] = (i % kHdrFloats) == kHdrMref ? -INFINITY : 0.f;
  }
  const SplitJob jb = js.job[blockIdx.y];
  const int nplanes = jb.nplanes;
  const float* sb = jb.src + size_t(blockIdx.x) * K * K;
  const int lk = 31 - __builtin_clz(unsigned(K));
  float hsc = 1.f;   // float16 job: the block's scale
  if (jb.fscale) {
    __shared__ float wmx[kSplitThreads / 64];
    float m = 0.f;
    for (int e = threadIdx.x * 4; e < K * K; e += kSplitThreads * 4) {
      const float4 v = *reinterpret_cast<const float4*>(sb + e);
      m = fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
    m = cluster_allmax<64>(m);
    if ((threadIdx.x & 63) == 0) wmx[threadIdx.x >> 6] = m;
    __syncthreads();
    m = 0.f;
    for (int i = 0; i < kSplitThreads / 64; ++i) m = fmaxf(m, wmx[i]);
    int ex = int(__float_as_uint(m) >> 23);
    ex = ex < 32 ? 32 : (ex > 254 ? 254 : ex);
    hsc = __uint_as_float(uint32_t(254 + jb.texp - ex) << 23);             // 2^(texp - (ex - 127))
    if (threadIdx.x == 0 && blockIdx.z == 0) jb.fscale[blockIdx.x] = __uint_as_float(uint32_t(ex - jb.texp) << 23);
  }
  // (grid z: with few blocks the stages of a block are dealt out to several workgroups)
  for (int stage = blockIdx.z; stage < nst; stage += gridDim.z) {
    uint16_t* buf = lds;
    uint16_t* db = jb.dst + (size_t(blockIdx.x) * nst + stage) * nplanes * K * 32;
    // a thread takes four inputs that are adjacent in the plane (e = 0..3 of one (row, step, half, u)):
    // one 128-bit load (or four coalesced loads of a transposed source) and one 64-bit LDS store per plane
    for (int qd = threadIdx.x; qd < K * 8; qd += kSplitThreads) {
      int out, wq;
      float x[4];
      if (jb.trans) {
        out = qd & (K - 1); wq = qd >> lk;
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = sb[size_t(32 * stage + 4 * wq + e) * K + out];
      } else {
        out = qd >> 3; wq = qd & 7;
        const float4 v = *reinterpret_cast<const float4*>(sb + size_t(out) * K + 32 * stage + 4 * wq);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
      }
      // quad wq holds inputs 4 wq .. 4 wq + 3 of the stage = 16 c2 + 8 u + 4 hh + e; with the natural order the
      // lane half takes eight consecutive inputs, i.e. the two middle bits swap their roles
      const int c2 = wq >> 2, u = jb.natural ? (wq & 1) : (wq >> 1) & 1, hh = jb.natural ? (wq >> 1) & 1 : (wq & 1);
      const int chunk = (2 * c2 + hh) ^ ((out >> 2) & 3);
      const int at = out * 32 + chunk * 8 + 4 * u;
      if (jb.fscale) {
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float y = x[e] * hsc;
          const _Float16 a = _Float16(y);
          const _Float16 b = _Float16(y - float(a));
          hi[e] = __builtin_bit_cast(uint16_t, a);
          lo[e] = __builtin_bit_cast(uint16_t, b);
        }
        *reinterpret_cast<uint2*>(buf + at) = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
        *reinterpret_cast<uint2*>(buf + at + K * 32) = make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
        continue;
      }
      for (int pl = 0; pl < nplanes; ++pl) {
        uint32_t part[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint32_t bits = __float_as_uint(x[e]);
          bits += 0x7FFFu + ((bits >> 16) & 1u);          // round to nearest even
          part[e] = bits >> 16;
          x[e] -= __uint_as_float(part[e] << 16);
        }
        *reinterpret_cast<uint2*>(buf + at + pl * K * 32) = make_uint2(part[0] | (part[1] << 16), part[2] | (part[3] << 16));
      }
    }
    __syncthreads();
    const uint4* s4 = reinterpret_cast<const uint4*>(buf);
    uint4* d4 = reinterpret_cast<uint4*>(db);
    for (int e = threadIdx.x; e < nplanes * K * 4; e += kSplitThreads) d4[e] = s4[e];
    __syncthreads();   // drained before the next stage overwrites it
  }
}

// rG[gi] = sum of rho over the axis indices of group gi (axis index a -> block (a/K)/rep, a%K).
// One wave per group.
__global__ __launch_bounds__(256) void rho_group_kernel(const float* __restrict__ rho, int K, int rep,
                                                         int G, int64_t ngroups, float* __restrict__ rG) {
  const int64_t gi = int64_t(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (gi >= ngroups) return;
  const int lane = threadIdx.x % kWave;
  float acc = 0.f;
  for (int e = lane; e < G; e += kWave) {
    const int64_t a = gi * G + e;
    acc += rho[((a / K) / rep) * K + a % K];
  }
  acc = wave_sum(acc);
  if (lane == 0) rG[gi] = acc;
}

// ---------------------------------------------------------------------------------------
// reduction of the per-(workgroup, segment) partials
// ---------------------------------------------------------------------------------------
// workgroups whose chunk of macro-tiles intersects segment `seg`: [lo, hi)
__device__ void seg_wg_range(int64_t seg, int64_t mt_per_seg, int64_t n_mt, int nwg, int* lo, int* hi) {
  const int64_t t0 = seg * mt_per_seg, t1 = t0 + mt_per_seg;
  int a = int((t0 * nwg) / n_mt);
  while (a > 0 && chunk_begin(a, n_mt, nwg) > t0) --a;
  while (a + 1 < nwg && chunk_begin(a + 1, n_mt, nwg) <= t0) ++a;
  int b = a;
  while (b < nwg && chunk_begin(b, n_mt, nwg) < t1) ++b;
  *lo = a;
  *hi = b;
}

struct ReduceArgs {
  const float* slot_grad;
  const float* slot_hdr;
  int64_t mt_per_seg, n_mt;   // of the pass that wrote the partials
  int nwg, nseg;
  int K, rep;
  int seg_len;           // axis indices per segment of that pass
  int part_floats;       // floats of one partial
  int msplit;            // 1: a partial holds whole blocks, [seg_len outputs][K inputs];
                         // 2: K == 256 in halves of the inputs, [256 outputs][128 inputs], segment 2 q + half
  int transpose_out;     // 1: out[m][j] = acc[j][m]
  float t;               // kLossLse: temperature; scale of a partial = exp(t (m_ref - m*)) / S
  const double* lse_ms;  // kLossLse: [0] = m*, [1] = S  (null for kLossSur)
  const float* member_ref;  // kLossLse, two-pass gradient: every partial is relative to this value
  float* out;            // [nb][K][K]
};

// grid: (nb transform blocks, K*K/1024).  out_b = sum over the rep row-blocks q of block b, and
// over the partials of q's segment, in fixed order; each thread owns four consecutive inputs of one
// output row, each workgroup 1024 elements that lie in one partial layout (one half when msplit == 2).
struct ReduceJobs { ReduceArgs job[2]; };   // grid.z picks the job (the two members of a pair in one launch)
__device__ __forceinline__ void reduce_grad_body(const ReduceArgs& a, const int b, const int by) {
  constexpr int kBatch = 64;
  __shared__ const float* src[kBatch];
  __shared__ float scl[kBatch];
  __shared__ int rng_lo, rng_hi;
  const int K = a.K;
  // this workgroup's 1024 elements: rows of KMr inputs inside one half
  const int KMr = a.msplit == 2 ? 128 : K;
  const int rows_per_wg = 1024 / KMr;                       // K = 32: one workgroup covers the block
  const int nyh = K / rows_per_wg > 0 ? K / rows_per_wg : 1;
  const int half = by / nyh, rg = by % nyh;
  const int j = rg * rows_per_wg + (threadIdx.x * 4) / KMr, ml = (threadIdx.x * 4) % KMr;
  const bool active = j < K;
  const int poff = j * KMr + ml;                            // offset inside a partial (plus the block's base)
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  // every partial of a two-pass member carries the same scale
  float sc_all = 1.f;
  if (a.lse_ms && a.member_ref) sc_all = float(exp(double(a.t) * (double(*a.member_ref) - a.lse_ms[0])) / a.lse_ms[1]);
  for (int q = b * a.rep; q < (b + 1) * a.rep; ++q) {
    int seg, base;
    if (a.msplit == 2) { seg = 2 * q + half; base = 0; }
    else { seg = int((int64_t(q) * K) / a.seg_len); base = int((int64_t(q) * K) % a.seg_len) * K; }
    if (threadIdx.x == 0) {
      int lo, hi;
      seg_wg_range(seg, a.mt_per_seg, a.n_mt, a.nwg, &lo, &hi);
      rng_lo = lo; rng_hi = hi;
    }
    __syncthreads();
    const int lo = rng_lo, hi = rng_hi;
    for (int w0 = lo; w0 < hi; w0 += kBatch) {
      const int n = hi - w0 < kBatch ? hi - w0 : kBatch;
      // the list of (partial, scale) pairs of this batch, one thread per entry
      if (int(threadIdx.x) < n) {
        const int64_t slot = int64_t(w0 + int(threadIdx.x)) + seg;
        float sc = sc_all;
        if (a.lse_ms && !a.member_ref)
          sc = float(exp(double(a.t) * (double(a.slot_hdr[slot * kHdrFloats + kHdrMref]) - a.lse_ms[0])) / a.lse_ms[1]);
        src[threadIdx.x] = a.slot_grad + slot * int64_t(a.part_floats) + base;
        scl[threadIdx.x] = sc;
      }
      __syncthreads();
      if (active) {
        // four partials in flight per thread; the additions keep the order of the list
        int s = 0;
        for (; s + 4 <= n; s += 4) {
          float4 v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(src[s + u] + poff);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float sc = scl[s + u];
            acc.x += sc * v[u].x; acc.y += sc * v[u].y; acc.z += sc * v[u].z; acc.w += sc * v[u].w;
          }
        }
        for (; s < n; ++s) {
          const float4 v = *reinterpret_cast<const float4*>(src[s] + poff);
          const float sc = scl[s];
          acc.x += sc * v.x; acc.y += sc * v.y; acc.z += sc * v.z; acc.w += sc * v.w;
        }
      }
      __syncthreads();
    }
  }
  if (active) {
    float* dst = a.out + size_t(b) * K * K;
    const int m = half * 128 + ml;
    if (a.transpose_out) {
      dst[(m + 0) * K + j] = acc.x; dst[(m + 1) * K + j] = acc.y;
      dst[(m + 2) * K + j] = acc.z; dst[(m + 3) * K + j] = acc.w;
    } else {
      *reinterpret_cast<float4*>(dst + j * K + m) = acc;
    }
  }
}
__global__ __launch_bounds__(256) void reduce_grad_kernel(const ReduceJobs js) {
  reduce_grad_body(js.job[blockIdx.z], int(blockIdx.x), int(blockIdx.y));
}

// v[axis index] = beta * sum over partials of the group's sum a^2, expanded per index, then
// Mmid_b = diag(v_b) P_b (scale_rows) or P_b diag(v_b).  For AXIS_ROW with rep > 1 the rep
// row-blocks of a transform block add up.   grid: nb transform blocks.
struct VArgs {
  const float* slot_hdr;
  int64_t mt_per_seg, n_mt;
  int nwg;
  int K, L, G, rep;
  float beta;
  const float* P;
  int scale_rows;
  float* Mmid;
};
constexpr int kMmidParts = 4;   // workgroups per block in the middle factor of the rho path
// (part of nparts: the workgroup scales that share of the block's elements; every part forms the same sums)
__device__ __forceinline__ void build_mmid_body(const VArgs& a, const int b, const int part, const int nparts) {
  __shared__ float v[256];
  __shared__ int rng[2];
  const int K = a.K, n = threadIdx.x;   // K <= 256 = blockDim.x: thread n owns index n
  double acc = 0;
  for (int q = b * a.rep; q < (b + 1) * a.rep; ++q) {
    // the K axis indices of a row-block lie in one segment (L is a multiple of K): its range of
    // workgroups is found once (64-bit divisions) and shared
    const int64_t seg = (int64_t(q) * K) / a.L;
    if (n == 0) {
      int lo, hi;
      seg_wg_range(seg, a.mt_per_seg, a.n_mt, a.nwg, &lo, &hi);
      rng[0] = lo; rng[1] = hi;
    }
    __syncthreads();
    const int lo = rng[0], hi = rng[1];
    if (n < K) {
      const int gi = int(((int64_t(q) * K + n) % a.L) / a.G);
      const float* h0 = a.slot_hdr + seg * kHdrFloats + kHdrVa2 + gi;
      // eight requests in flight; the additions keep the order of the workgroups
      int w = lo;
      for (; w + 8 <= hi; w += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = h0[int64_t(w + u) * kHdrFloats];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += t[u];
      }
      for (; w < hi; ++w) acc += h0[int64_t(w) * kHdrFloats];
    }
    __syncthreads();
  }
  if (n < K) v[n] = float(acc * a.beta);
  __syncthreads();
  const float* Pb = a.P + size_t(b) * K * K;
  float* Mb = a.Mmid + size_t(b) * K * K;
  // K * K / nparts elements, four per thread and step (K is a multiple of 32: rows are multiples of 4)
  const int per = K * K / nparts, e0 = part * per;
  for (int i = e0 + 4 * int(threadIdx.x); i < e0 + per; i += 4 * int(blockDim.x)) {
    const float4 pv = *reinterpret_cast<const float4*>(Pb + i);
    float4 o;
    if (a.scale_rows) {
      const float f = v[i / K];
      o = make_float4(pv.x * f, pv.y * f, pv.z * f, pv.w * f);
    } else {
      const int c = i % K;
      o = make_float4(pv.x * v[c], pv.y * v[c + 1], pv.z * v[c + 2], pv.w * v[c + 3]);
    }
    *reinterpret_cast<float4*>(Mb + i) = o;
  }
}
__global__ __launch_bounds__(256) void build_mmid_kernel(const VArgs a) {
  build_mmid_body(a, int(blockIdx.x) / kMmidParts, int(blockIdx.x) % kMmidParts, kMmidParts);
}

// losses: fixed-order float64 sums over every partial header (loss_reduce.hpp), as a launch of its own
__global__ __launch_bounds__(kLossThreads) void reduce_losses_kernel(const LossArgs a) {
  __shared__ double red[5 * (kLossThreads / 64)];
  double m, s;
  reduce_losses_body<kLossThreads>(a, red, true, &m, &s);
}

// What follows the loss / gradient kernel of a single matrix whose gradient comes as partials, in one launch:
// the gradient reduction (nred_x x nred_y workgroups), the middle factor of the gradient's way through rho(P)
// (kMmidParts workgroups per block) and the loss reduction (one workgroup) read the same partials and do not depend
// on each other.
__global__ __launch_bounds__(256) void single_tail_kernel(const ReduceArgs ra, const VArgs va, const LossArgs la,
                                                          const int nred_x, const int nred_y, const int nb) {
  const int id = int(blockIdx.x), nred = nred_x * nred_y;
  if (id < nred) {
    reduce_grad_body(ra, id % nred_x, id / nred_x);
  } else if (id < nred + nb * kMmidParts) {
    build_mmid_body(va, (id - nred) / kMmidParts, (id - nred) % kMmidParts, kMmidParts);
  } else {
    __shared__ double red[5 * (kLossThreads / 64)];
    double m, sm;
    reduce_losses_body<kLossThreads>(la, red, true, &m, &sm);
  }
}

// ---------------------------------------------------------------------------------------
// batched k x k product  C_b = alpha * op(A_b) op(B_b) + beta * C_b   (64 x 64 tile / workgroup)
// ---------------------------------------------------------------------------------------
template <bool TA, bool TB>
__global__ __launch_bounds__(256) void bgemm_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                     float* __restrict__ C, int K, float alpha, float beta) {
  __shared__ float sa[16][68];   // [l][i]
  __shared__ float sb[16][68];   // [l][j]
  const int tpr = K / 64;
  const int b = blockIdx.x / (tpr * tpr), tile = blockIdx.x % (tpr * tpr);
  const int i0 = (tile / tpr) * 64, j0 = (tile % tpr) * 64;
  const float* Ab = A + size_t(b) * K * K;
  const float* Bb = B + size_t(b) * K * K;
  float* Cb = C + size_t(b) * K * K;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int l0 = 0; l0 < K; l0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      const int l = e / 64, i = e % 64;
      sa[l][i] = TA ? Ab[(l0 + l) * K + i0 + i] : Ab[(i0 + i) * K + l0 + l];
      sb[l][i] = TB ? Bb[(j0 + i) * K + l0 + l] : Bb[(l0 + l) * K + j0 + i];
    }
    __syncthreads();
#pragma unroll
    for (int l = 0; l < 16; ++l) {
      float av[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { av[u] = sa[l][ty * 4 + u]; bv[u] = sb[l][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(av[u], bv[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float* dst = Cb + (i0 + ty * 4 + u) * K + j0 + tx * 4 + v;
      *dst = alpha * acc[u][v] + (beta != 0.f ? beta * *dst : 0.f);
    }
}

// Same product on the matrix cores (v_mfma_f32_32x32x2_f32) for K a multiple of 64: one 64 x 64
// output tile per workgroup, four waves of one 32 x 32 tile each, the operand panels staged in
// LDS as [contraction index][64 tile indices] (row stride 65 floats: transposing stores, whose
// lanes walk the contraction index, and the MFMA operand reads, whose lane halves take rows l
// and l+1, both stay clear of bank conflicts).  Contraction in chunks of CH = min(K, 128): the blocks of
// 128 the learning loops run on take one chunk -- every load of the workgroup is in flight at once and
// there is one barrier -- at 65 KB of LDS, two workgroups per compute unit.
template <bool TA, bool TB, int CH>
// D: where the beta term is read (null: C itself); skip: optional per-block flags, a block whose flag is set is
// left alone.
__global__ __launch_bounds__(256) void bgemm_mfma_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                          float* __restrict__ C, int K, float alpha, float beta,
                                                          const AdamHook adam, const float* __restrict__ D,
                                                          const int* __restrict__ skip) {
  constexpr int LD = 65;
  extern __shared__ __align__(16) float bsm[];
  float* sa = bsm;
  float* sb = bsm + CH * LD;
  const int tpr = K / 64;
  const int b = blockIdx.x / (tpr * tpr), tile = blockIdx.x % (tpr * tpr);
  if (skip && skip[b]) return;
  const int i0 = (tile / tpr) * 64, j0 = (tile % tpr) * 64;
  const float* Ab = A + size_t(b) * K * K;
  const float* Bb = B + size_t(b) * K * K;
  float* Cb = C + size_t(b) * K * K;
  const float* Db = (D ? D : C) + size_t(b) * K * K;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, h = lane >> 5;
  const int wi = wave >> 1, wj = wave & 1;
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  // the old value of the output, where it is added to: requested before everything else
  float cold[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) cold[v] = 0.f;
  if (beta != 0.f) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      cold[v] = Db[(i0 + wi * 32 + 8 * (v / 4) + 4 * h + (v % 4)) * K + j0 + wj * 32 + ln];
  }
  for (int l0 = 0; l0 < K; l0 += CH) {
    // sa[l][i] = op(A)[i0 + i][l0 + l];  sb[l][j] = op(B)[l0 + l][j0 + j]: four consecutive elements of the
    // operand's rows per load, all loads of the chunk issued before the first LDS store
    constexpr int NV = CH * 64 / 4 / 256;   // float4 per thread and panel
    float4 va[NV], vb[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int e = (tid + u * 256) * 4;
      if (TA) { const int l = e >> 6, i = e & 63; va[u] = *reinterpret_cast<const float4*>(Ab + (l0 + l) * K + i0 + i); }
      else    { const int i = e / CH, l = e % CH; va[u] = *reinterpret_cast<const float4*>(Ab + (i0 + i) * K + l0 + l); }
      if (TB) { const int j = e / CH, l = e % CH; vb[u] = *reinterpret_cast<const float4*>(Bb + (j0 + j) * K + l0 + l); }
      else    { const int l = e >> 6, j = e & 63; vb[u] = *reinterpret_cast<const float4*>(Bb + (l0 + l) * K + j0 + j); }
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int e = (tid + u * 256) * 4;
      if (TA) { const int l = e >> 6, i = e & 63; float* d = sa + l * LD + i; d[0] = va[u].x; d[1] = va[u].y; d[2] = va[u].z; d[3] = va[u].w; }
      else    { const int i = e / CH, l = e % CH; float* d = sa + l * LD + i; d[0] = va[u].x; d[LD] = va[u].y; d[2 * LD] = va[u].z; d[3 * LD] = va[u].w; }
      if (TB) { const int j = e / CH, l = e % CH; float* d = sb + l * LD + j; d[0] = vb[u].x; d[LD] = vb[u].y; d[2 * LD] = vb[u].z; d[3 * LD] = vb[u].w; }
      else    { const int l = e >> 6, j = e & 63; float* d = sb + l * LD + j; d[0] = vb[u].x; d[1] = vb[u].y; d[2] = vb[u].z; d[3] = vb[u].w; }
    }
    __syncthreads();
    const float* pa = sa + h * LD + wi * 32 + ln;
    const float* pb = sb + h * LD + wj * 32 + ln;
    for (int s0 = 0; s0 < CH / 2; s0 += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * (s0 + u) * LD], pb[2 * (s0 + u) * LD], acc, 0, 0, 0);
    }
    if (l0 + CH < K) __syncthreads();
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = i0 + wi * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = j0 + wj * 32 + ln;
    const float g = alpha * acc[v] + (beta != 0.f ? beta * cold[v] : 0.f);
    if (adam.T) {
      // (the arithmetic of adam_kernel, on the gradient still in its register)
      const size_t at = size_t(b) * K * K + size_t(i) * K + j;
      const float mi = adam.beta1 * adam.m[at] + adam.omb1 * g;
      const float vi = adam.beta2 * adam.v[at] + adam.omb2 * g * g;
      adam.m[at] = mi;
      adam.v[at] = vi;
      adam.T[at] -= adam.lr * (mi * adam.c1) / (sqrtf(vi * adam.c2) + adam.eps);
    } else {
      Cb[i * K + j] = g;
    }
  }
}

// The gradient's way through the inverse in one launch for blocks of 128: C = beta C + alpha (P^T G) P^T per block
// (Sec. 4.1 / 4.2: d/dT of a function of P = T^-1 is -P^T (d/dP) P^T).  Row i of the result needs row i of
// X = P^T G only, so a workgroup that owns 64 rows computes its slice of X and then its slice of X P^T with no
// exchange between workgroups: two workgroups per block, eight waves of one 32 x 32 tile each, both products on
// v_mfma_f32_32x32x2_f32 in the arithmetic (and summation order) of bgemm_mfma_kernel.  P is staged once in LDS,
// row-major with a row stride of 129 floats, which serves the first product's A operand (lanes along a row) and
// the second's B operand (lanes along a column) without bank conflicts; G goes from memory straight into the
// registers of the wave that multiplies by it; X passes through LDS transposed.
// (Blocks of 64: one workgroup of four waves per block, the same scheme.)
constexpr int kChainLdX = 33;
constexpr size_t chain_lds(int K) { return size_t(K * (K + 1) + 2 * K * kChainLdX) * sizeof(float); }
template <int K>
__global__ __launch_bounds__(4 * K) void bgemm_chain_kernel(const float* __restrict__ P, const float* __restrict__ G,
                                                            float* __restrict__ C, float alpha, float beta,
                                                            const AdamHook adam) {
  static_assert(K == 64 || K == 128, "slices of 64 rows");
  constexpr int kChainLdP = K + 1, NT = 4 * K, WJ = K / 32, SL = K / 64;   // threads, column tiles, slices per block
  extern __shared__ __align__(16) float csm[];
  float* sp = csm;                          // P[r][c]
  float* sx = csm + K * kChainLdP;          // [2 row halves][l][32 rows]: X^T of the workgroup's slice
  const int b = blockIdx.x / SL, i0 = (blockIdx.x % SL) * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, h = lane >> 5;
  const int wi = wave / WJ, wj = wave % WJ;
  const float* Pb = P + size_t(b) * K * K;
  const float* Gb = G + size_t(b) * K * K;
  float* Cb = C + size_t(b) * K * K;
  // every load of the workgroup is requested before the first wait: P (for LDS), this wave's columns of G, and the
  // old value of the output where it is added to
  constexpr int NVP = K * K / 4 / NT;       // float4 of P per thread
  float4 vp[NVP];
#pragma unroll
  for (int u = 0; u < NVP; ++u) vp[u] = *reinterpret_cast<const float4*>(Pb + (tid + u * NT) * 4);
  float g[K / 2];
#pragma unroll
  for (int t = 0; t < K / 2; ++t) g[t] = Gb[(2 * t + h) * K + wj * 32 + ln];
  float cold[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) cold[v] = 0.f;
  if (beta != 0.f) {
#pragma unroll
    for (int v = 0; v < 16; ++v) cold[v] = Cb[(i0 + wi * 32 + 8 * (v / 4) + 4 * h + (v % 4)) * K + wj * 32 + ln];
  }
#pragma unroll
  for (int u = 0; u < NVP; ++u) {
    const int e = (tid + u * NT) * 4, r = e / K, c = e % K;
    float* d = sp + r * kChainLdP + c;
    d[0] = vp[u].x; d[1] = vp[u].y; d[2] = vp[u].z; d[3] = vp[u].w;
  }
  __syncthreads();
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  {
    // X[i][j] = sum_l P[l][i] G[l][j]
    const float* pa = sp + h * kChainLdP + i0 + wi * 32 + ln;
#pragma unroll
    for (int t = 0; t < K / 2; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * t * kChainLdP], g[t], acc, 0, 0, 0);
  }
  {
    float* xw = sx + wi * (K * kChainLdX) + (wj * 32 + ln) * kChainLdX;
#pragma unroll
    for (int v = 0; v < 16; ++v) xw[8 * (v / 4) + 4 * h + (v % 4)] = acc[v];
  }
  __syncthreads();
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  {
    // Y[i][j] = sum_l X[i][l] P[j][l]
    const float* pa = sx + wi * (K * kChainLdX) + h * kChainLdX + ln;
    const float* pb = sp + (wj * 32 + ln) * kChainLdP + h;
#pragma unroll 8
    for (int t = 0; t < K / 2; ++t)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * t * kChainLdX], pb[2 * t], acc, 0, 0, 0);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = i0 + wi * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = wj * 32 + ln;
    const float gr = alpha * acc[v] + (beta != 0.f ? beta * cold[v] : 0.f);
    if (adam.T) {
      // (the arithmetic of adam_kernel, on the gradient still in its register)
      const size_t at = size_t(b) * K * K + size_t(i) * K + j;
      const float mi = adam.beta1 * adam.m[at] + adam.omb1 * gr;
      const float vi = adam.beta2 * adam.v[at] + adam.omb2 * gr * gr;
      adam.m[at] = mi;
      adam.v[at] = vi;
      adam.T[at] -= adam.lr * (mi * adam.c1) / (sqrtf(vi * adam.c2) + adam.eps);
    } else {
      Cb[i * K + j] = gr;
    }
  }
}


// K == 32: one 32 x 32 tile per workgroup, thread per output element group
template <bool TA, bool TB>
__global__ __launch_bounds__(256) void bgemm32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       float* __restrict__ C, float alpha, float beta) {
  constexpr int K = 32;
  __shared__ float sa[K][K + 1], sb[K][K + 1];
  const float* Ab = A + size_t(blockIdx.x) * K * K;
  const float* Bb = B + size_t(blockIdx.x) * K * K;
  float* Cb = C + size_t(blockIdx.x) * K * K;
  for (int e = threadIdx.x; e < K * K; e += 256) {
    const int r = e / K, c = e % K;
    sa[r][c] = TA ? Ab[c * K + r] : Ab[e];   // sa[i][l]
    sb[r][c] = TB ? Bb[c * K + r] : Bb[e];   // sb[l][j]
  }
  __syncthreads();
  for (int e = threadIdx.x; e < K * K; e += 256) {
    const int i = e / K, j = e % K;
    float acc = 0.f;
#pragma unroll
    for (int l = 0; l < K; ++l) acc = fmaf(sa[i][l], sb[l][j], acc);
    Cb[e] = alpha * acc + (beta != 0.f ? beta * Cb[e] : 0.f);
  }
}

}  // namespace

int launch_split_planes_multi(const SplitRequest* req, int n, int K, int nb, hipStream_t st, float* hdr,
                              int64_t nslot) {
  SplitJobs js;
  js.njobs = n; js.K = K; js.hdr = hdr; js.nhdr = nslot * kHdrFloats;
  for (int i = 0; i < n && i < 4; ++i) {
    js.job[i].src = req[i].src; js.job[i].dst = req[i].dst;
    js.job[i].trans = req[i].trans; js.job[i].nplanes = req[i].fscale ? 2 : req[i].nplanes;
    js.job[i].fscale = req[i].fscale; js.job[i].natural = req[i].natural; js.job[i].texp = req[i].texp;
  }
  // one workgroup per (block, job) when those fill the chip; else one per (block, job, stage)
  const int zsplit = nb * n >= 128 ? 1 : K / 32;
  hipLaunchKernelGGL(split_planes_kernel, dim3(nb, n, zsplit), dim3(kSplitThreads), 0, st, js);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_split_planes(const float* src, int K, int nb, int trans, int nplanes, uint16_t* dst, hipStream_t st) {
  SplitRequest r{src, dst, trans, nplanes};
  return launch_split_planes_multi(&r, 1, K, nb, st);
}
// Whether launch_rho can also form the group sums of rho_group_kernel for groups of G axis indices.
bool rho_groups_inline(int K, int nb, int G, int rep) {
  if (G >= 1 && G <= K) return K % G == 0;
  return rep == 1 && G <= 256 && G % K == 0 && nb % (G / K) == 0;
}
int launch_rho(const float* P, int K, int nb, int by_row, float* rho, hipStream_t st, float* rG, int G, int rep) {
  if (rG && !rho_groups_inline(K, nb, G, rep)) return CAFEQ_ERR_INVALID_ARG;
  const int nbk = rG && G > K ? G / K : 1;
  hipLaunchKernelGGL(rho_kernel, dim3(nb / nbk), dim3(256), 0, st, P, K, by_row, rho, rG, G, rep, nbk);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_rho_groups(const float* rho, int K, int rep, int G, int64_t ngroups, float* rG, hipStream_t st) {
  hipLaunchKernelGGL(rho_group_kernel, dim3(unsigned((ngroups + 3) / 4)), dim3(256), 0, st, rho, K, rep, G,
                     ngroups, rG);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
namespace {
// fused: the partials were written by the fused kernel (segments of max(K, G), [NBLK][K][K]); otherwise by the
// gradient pass (chunks of 128 inputs; halves of the inputs for K == 256)
ReduceArgs reduce_args(const CoreParams& p, int K, int G, bool fused, int transpose_out, const double* lse_ms,
                       const float* member_ref, float* out) {
  ReduceArgs a;
  a.slot_grad = p.slot_grad; a.slot_hdr = p.slot_hdr; a.mt_per_seg = p.mt_per_seg; a.n_mt = p.n_mt;
  a.nwg = p.nwg; a.nseg = p.nseg; a.K = K; a.rep = p.rep;
  if (fused) {
    const int L = K > G ? K : G;
    a.seg_len = L; a.part_floats = L * K; a.msplit = 1;
  } else {
    a.seg_len = 128; a.msplit = K == 256 ? 2 : 1; a.part_floats = K == 256 ? 256 * 128 : 128 * K;
  }
  a.transpose_out = transpose_out; a.t = p.lse_t; a.lse_ms = lse_ms; a.member_ref = member_ref; a.out = out;
  return a;
}
}  // namespace
int launch_reduce_grad(const CoreParams& p, int K, int G, bool fused, int nb, int transpose_out,
                       const double* lse_ms, const float* member_ref, float* out, hipStream_t st) {
  ReduceJobs js;
  js.job[0] = js.job[1] = reduce_args(p, K, G, fused, transpose_out, lse_ms, member_ref, out);
  hipLaunchKernelGGL(reduce_grad_kernel, dim3(nb, (K * K + 1023) / 1024, 1), dim3(256), 0, st, js);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
// Both members of a pair in one launch: pa -> outA (transposed), pb -> outB.
int launch_reduce_grad_pair(const CoreParams& pa, int GA, bool fusedA, const float* refA, float* outA,
                            const CoreParams& pb, int GB, bool fusedB, const float* refB, float* outB, int K,
                            int nb, const double* lse_ms, hipStream_t st) {
  ReduceJobs js;
  js.job[0] = reduce_args(pa, K, GA, fusedA, 1, lse_ms, refA, outA);
  js.job[1] = reduce_args(pb, K, GB, fusedB, 0, lse_ms, refB, outB);
  hipLaunchKernelGGL(reduce_grad_kernel, dim3(nb, (K * K + 1023) / 1024, 2), dim3(256), 0, st, js);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_build_mmid(const CoreParams& p, int K, int G, int nb, const float* P, int scale_rows, float* Mmid,
                      hipStream_t st) {
  VArgs a;
  a.slot_hdr = p.slot_hdr; a.mt_per_seg = p.mt_per_seg; a.n_mt = p.n_mt; a.nwg = p.nwg;
  a.K = K; a.L = K > G ? K : G; a.G = G; a.rep = p.rep; a.beta = p.beta; a.P = P;
  a.scale_rows = scale_rows; a.Mmid = Mmid;
  hipLaunchKernelGGL(build_mmid_kernel, dim3(nb * kMmidParts), dim3(256), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_single_tail(const CoreParams& pgrad, const CoreParams& ploss, int K, int G, bool fused, int nb,
                       int transpose_out, float* gradT, const float* P, int scale_rows, float* Mmid, float beta,
                       int nslot, float* losses, double* lse_ms, hipStream_t st) {
  const ReduceArgs ra = reduce_args(pgrad, K, G, fused, transpose_out, nullptr, nullptr, gradT);
  VArgs va;
  va.slot_hdr = ploss.slot_hdr; va.mt_per_seg = ploss.mt_per_seg; va.n_mt = ploss.n_mt; va.nwg = ploss.nwg;
  va.K = K; va.L = K > G ? K : G; va.G = G; va.rep = ploss.rep; va.beta = ploss.beta; va.P = P;
  va.scale_rows = scale_rows; va.Mmid = Mmid;
  LossArgs la{};
  la.hdrA = ploss.slot_hdr; la.nslotA = nslot; la.kind = kLossSur; la.beta = beta; la.losses = losses;
  la.lse_ms = lse_ms;
  const int nred_x = nb, nred_y = (K * K + 1023) / 1024;
  hipLaunchKernelGGL(single_tail_kernel, dim3(unsigned(nred_x * nred_y + nb * kMmidParts + 1)), dim3(256), 0, st, ra, va, la,
                     nred_x, nred_y, nb);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_reduce_losses(int kind, const float* hdrA, int nslotA, const float* hdrB, int nslotB, float beta,
                         float t, int64_t ngroups, float* losses, double* lse_ms, hipStream_t st) {
  LossArgs a;
  a.hdrA = hdrA; a.nslotA = nslotA; a.hdrB = hdrB; a.nslotB = nslotB; a.kind = kind; a.beta = beta; a.t = t;
  a.ngroups = ngroups; a.losses = losses; a.lse_ms = lse_ms;
  hipLaunchKernelGGL(reduce_losses_kernel, dim3(1), dim3(kLossThreads), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_bgemm(bool ta, bool tb, const float* A, const float* B, float* C, int K, int nb, float alpha,
                 float beta, hipStream_t st, const AdamHook* adam, const float* D, const int* skip) {
  AdamHook hook;
  hook.T = nullptr;
  if (adam) {
    if (K == 32) return CAFEQ_ERR_INVALID_ARG;
    hook = *adam;
  }
  if ((D || skip) && K == 32) return CAFEQ_ERR_INVALID_ARG;
  if (K == 32) {
#define CAFEQ_G32(TA, TB) hipLaunchKernelGGL((bgemm32_kernel<TA, TB>), dim3(nb), dim3(256), 0, st, A, B, C, alpha, beta)
    if (ta && tb) CAFEQ_G32(true, true); else if (ta) CAFEQ_G32(true, false);
    else if (tb) CAFEQ_G32(false, true); else CAFEQ_G32(false, false);
#undef CAFEQ_G32
  } else {
    const unsigned grid = unsigned(nb) * (K / 64) * (K / 64);
    if (K % 128 == 0) {
      constexpr int CH = 128;
      constexpr size_t lds = 2 * CH * 65 * sizeof(float);
      static std::atomic<bool> attr_set{false};
      if (!attr_set) {
        bool ok = true;
#define CAFEQ_ATTR(TA, TB)                                                                                     \
  ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(bgemm_mfma_kernel<TA, TB, CH>),                 \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) == hipSuccess
        CAFEQ_ATTR(true, true); CAFEQ_ATTR(true, false); CAFEQ_ATTR(false, true); CAFEQ_ATTR(false, false);
#undef CAFEQ_ATTR
        if (!ok) return CAFEQ_ERR_LAUNCH;
        attr_set = true;
      }
#define CAFEQ_G128(TA, TB) hipLaunchKernelGGL((bgemm_mfma_kernel<TA, TB, CH>), dim3(grid), dim3(256), lds, st, A, B, C, K, alpha, beta, hook, D, skip)
      if (ta && tb) CAFEQ_G128(true, true); else if (ta) CAFEQ_G128(true, false);
      else if (tb) CAFEQ_G128(false, true); else CAFEQ_G128(false, false);
#undef CAFEQ_G128
    } else {
      constexpr size_t lds = 2 * 64 * 65 * sizeof(float);
#define CAFEQ_G64(TA, TB) hipLaunchKernelGGL((bgemm_mfma_kernel<TA, TB, 64>), dim3(grid), dim3(256), lds, st, A, B, C, K, alpha, beta, hook, D, skip)
      if (ta && tb) CAFEQ_G64(true, true); else if (ta) CAFEQ_G64(true, false);
      else if (tb) CAFEQ_G64(false, true); else CAFEQ_G64(false, false);
#undef CAFEQ_G64
    }
  }
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
// C = beta C + alpha (P^T G) P^T per block; x1: scratch of nb K K floats for block sizes other than 128
int launch_bgemm_chain(const float* P, const float* G, float* x1, float* C, int K, int nb, float alpha, float beta,
                       hipStream_t st, const AdamHook* adam) {
  if (K != 128 && K != 64) {
    const int rc = launch_bgemm(true, false, P, G, x1, K, nb, 1.f, 0.f, st);
    if (rc) return rc;
    return launch_bgemm(false, true, x1, P, C, K, nb, alpha, beta, st, adam);
  }
  AdamHook hook;
  hook.T = nullptr;
  if (adam) hook = *adam;
  static std::atomic<bool> attr_set{false};
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(bgemm_chain_kernel<128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(chain_lds(128))) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(bgemm_chain_kernel<64>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(chain_lds(64))) != hipSuccess)
      return CAFEQ_ERR_LAUNCH;
    attr_set = true;
  }
  if (K == 128)
    hipLaunchKernelGGL(bgemm_chain_kernel<128>, dim3(unsigned(nb) * 2), dim3(512), chain_lds(128), st, P, G, C, alpha, beta, hook);
  else
    hipLaunchKernelGGL(bgemm_chain_kernel<64>, dim3(unsigned(nb)), dim3(256), chain_lds(64), st, P, G, C, alpha, beta, hook);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int device_cu_count() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cus = n;
  }
  return cus;
}

}  // namespace cafeq
