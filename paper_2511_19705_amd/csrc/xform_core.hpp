// Fused block-transform / quantize / inverse-transform / loss / gradient kernel (gfx950).
//
// Work decomposition.  A "line" is one vector along the transformed axis (a row of W for
// AXIS_COL, a column for AXIS_ROW).  The axis is cut into segments of L = max(K, G)
// elements (K: transform block, G: quantization group), so a segment holds whole blocks
// and whole groups.  One wavefront owns a strip of 32 lines x one segment:
//   Z^T[j][line] = sum_m Afwd[j][m] * W[line][m]         v_mfma_f32_32x32x2_f32
// with the transform tile as the MFMA A operand (from LDS) and the weights as the B
// operand, read from global memory straight into the lane that consumes them.  In the
// 32x32 accumulator layout a lane then holds, for ONE line, the axis indices
//   j(f, h) = 8*(f/4) + 4*h + f%4,   f = 0..L/2-1,  h = lane/32,
// so a group's absmax is a scan over registers plus one exchange with lane^32, the
// quantization error E replaces Z in the same registers, and -- because the MFMA B operand
// of lane (line, h) at step (c, s) is exactly element j(4c+s, h) -- those registers feed the
// inverse transform D^T = Ainv * E^T without any data movement.  Z, E and D never leave
// the register file; W is read from memory once.
//
// The transform tiles (32 outputs x K inputs, fp32) are streamed through a double-buffered
// LDS ring shared by the workgroup's waves (one barrier per tile step); they come from the
// L2, where the blocks of a segment stay resident while consecutive macro-tiles use them.
// Workgroups are persistent: each takes a contiguous range of macro-tiles (segment-major),
// keeps loss partial sums in registers and the dense k x k gradient accumulator in LDS
// (float atomics: lanes scatter rank-1 updates s * W[line][:] into row j* of the block), and
// writes one partial per (workgroup, segment) that a finishing kernel reduces in fixed order.
#pragma once
#include "cafeq_internal.hpp"

namespace cafeq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kNW = 4;              // waves per workgroup
constexpr int kThreads = kNW * 64;  // threads per workgroup
constexpr int kStripLines = 32;     // lines per wave
constexpr int kMacroLines = kNW * kStripLines;

__host__ __device__ constexpr int cmax(int a, int b) { return a > b ? a : b; }

template <int K, int G>
struct Geo {
  static constexpr int L = cmax(K, G);
  static constexpr int NBLK = L / K;      // transform blocks per segment
  static constexpr int NT = L / 32;       // 32-output tiles per segment
  static constexpr int KT = K / 32;       // tiles per block
  static constexpr int NGRP = L / G;      // groups per segment
  static constexpr int RPG = G / 2;       // accumulator registers per group per lane
  static constexpr int LDA = K + 4;       // LDS row stride of a transform tile (floats)
  static constexpr int RING_STAGES = 3;
  static constexpr int RING_FLOATS = RING_STAGES * 32 * LDA;
  static constexpr int GACC_FLOATS = NBLK * K * (K + 1);
  static constexpr int A_VEC_PER_THREAD = (32 * K / 4 + kThreads - 1) / kThreads;
};

// header layout of one partial (floats)
constexpr int kHdrL2 = 0, kHdrErrZ = 1, kHdrWsq = 2, kHdrSur = 3, kHdrMref = 4, kHdrVa2 = 8;
constexpr int kHdrFloats = 8 + 32;  // up to 32 groups per segment

enum : int { kLossSur = 0, kLossLse = 1 };

struct CoreParams {
  const void* W;
  int dtype;
  int64_t rows, cols, ld;
  const float* Afwd;  // [nb][K][K]; element [out][in], or [in][out] when afwd_trans
  const float* Ainv;  // [nb][K][K]; likewise with ainv_trans
  int afwd_trans, ainv_trans;
  int rep;            // AXIS_ROW: row-block q uses block q / rep
  int nseg;
  int64_t nlines;
  int64_t mt_per_seg, n_mt;
  int nwg;
  QGrid grid;
  int do_inverse, do_grad, loss_kind;
  float beta, lse_t;
  const float* rG;    // [nseg * NGRP] sum of rho over each group (kLossSur)
  float* Zout;        // optional outputs
  int8_t* codes;
  float* scales;
  float* slot_grad;   // [nwg + nseg][NBLK*K*K]
  float* slot_hdr;    // [nwg + nseg][kHdrFloats]
#ifdef CAFEQ_CORE_TIMING
  long long* dbg;     // [nwg][8] phase cycle counts of wave 0 (experiments only)
#endif
};

__device__ __forceinline__ int64_t chunk_begin(int64_t w, int64_t n_mt, int64_t nwg) {
  return (w * n_mt) / nwg;
}

// One 32 x K transform tile times the strip: 4 MFMAs per 128-bit LDS read, the reads issued
// one group (four reads) ahead of the MFMAs that consume them.  bop(i) is the B operand of
// MFMA i (i = 4*c + e uses input index 8c + 4h + e of the tile).
template <int K, typename BF>
__device__ __forceinline__ floatx16 tile_mfma(const float* abuf, BF bop) {
  constexpr int NC = K / 8, PF = 4, NG = NC / PF;
  floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float4 a[2][PF];
#pragma unroll
  for (int j = 0; j < PF; ++j) a[0][j] = *reinterpret_cast<const float4*>(abuf + 8 * j);
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) {
    if (gq + 1 < NG) {
#pragma unroll
      for (int j = 0; j < PF; ++j)
        a[(gq + 1) & 1][j] = *reinterpret_cast<const float4*>(abuf + 8 * ((gq + 1) * PF + j));
    }
    // keep the reads above this point: the scheduler otherwise sinks each read to just
    // before its first use and the matrix pipe idles for the whole LDS latency
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      const int c = gq * PF + j;
      const float4 v = a[gq & 1][j];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(v.x, bop(4 * c + 0), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(v.y, bop(4 * c + 1), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(v.z, bop(4 * c + 2), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(v.w, bop(4 * c + 3), acc, 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  return acc;
}

template <int K, int G, int AXIS>
__global__ __launch_bounds__(kThreads) void xform_core_kernel(const CoreParams p) {
  using g = Geo<K, G>;
  constexpr int L = g::L, NT = g::NT, KT = g::KT, NGRP = g::NGRP, RPG = g::RPG, LDA = g::LDA;
  constexpr int NBLK = g::NBLK;
  extern __shared__ __align__(16) float smem[];
  float* ring = smem;
  float* gacc = smem + g::RING_FLOATS;                                  // only if do_grad
  float* hred = gacc + (p.do_grad ? g::GACC_FLOATS : 0);                // [kNW][kHdrFloats]
  float* wmax = hred + kNW * kHdrFloats;                                // [kNW]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5;

  // contiguous chunks; consecutive chunks on the same XCD (workgroup i runs on XCD i % 8)
  int64_t w = blockIdx.x;
  if ((p.nwg & 7) == 0) w = int64_t(blockIdx.x & 7) * (p.nwg >> 3) + (blockIdx.x >> 3);
  const int64_t mt0 = chunk_begin(w, p.n_mt, p.nwg), mt1 = chunk_begin(w + 1, p.n_mt, p.nwg);
  if (mt0 >= mt1) return;

  const int tiles_per_mt = p.do_inverse ? 2 * NT : NT;
  const int total_tiles = int(mt1 - mt0) * tiles_per_mt;

  // The transform tiles are consumed in a fixed order: for each macro-tile, the NT forward
  // tiles then (loss calls) the NT inverse tiles of its segment.  A tile is the 32 x K slab
  // [32 outputs][K inputs] of one transform block.  Stored [out][in] it is contiguous; stored
  // [in][out] (the caller's T used as T^T) it is a 32-column stripe, transposed on its way
  // into LDS.  The fetch cursor runs two tiles ahead of the consumer and advances without
  // divisions.
  const int seg_first = int(mt0 / p.mt_per_seg);
  const int mis_first = int(mt0 - int64_t(seg_first) * p.mt_per_seg);   // macro-tile within segment
  const int mt_per_seg = int(p.mt_per_seg);
  int f_tau = 0, f_seg = seg_first, f_mis = mis_first;   // fetch cursor
  float4 areg[g::A_VEC_PER_THREAD];
  bool areg_trans = false;
  auto tile_fetch_next = [&]() {
    int tau = f_tau;
    const float* base = p.Afwd;
    areg_trans = p.afwd_trans != 0;
    if (tau >= NT) { tau -= NT; base = p.Ainv; areg_trans = p.ainv_trans != 0; }
    const int blk = f_seg * NBLK + tau / KT;
    const int b = (AXIS == CAFEQ_AXIS_ROW && p.rep != 1) ? blk / p.rep : blk;
    const int t32 = tau % KT;
    if (!areg_trans) {
      const float4* src = reinterpret_cast<const float4*>(base + (int64_t(b) * K + t32 * 32) * K);
#pragma unroll
      for (int i = 0; i < g::A_VEC_PER_THREAD; ++i) {
        const int id = tid + i * kThreads;
        if (id < 32 * K / 4) areg[i] = src[id];
      }
    } else {
      const float* src = base + int64_t(b) * K * K + t32 * 32;
#pragma unroll
      for (int i = 0; i < g::A_VEC_PER_THREAD; ++i) {
        const int id = tid + i * kThreads;       // input row m = id / 8, four outputs 4*(id % 8)..
        if (id < 32 * K / 4) areg[i] = *reinterpret_cast<const float4*>(src + (id >> 3) * K + 4 * (id & 7));
      }
    }
    if (++f_tau == tiles_per_mt) {
      f_tau = 0;
      if (++f_mis == mt_per_seg) { f_mis = 0; ++f_seg; }
    }
  };
  auto tile_commit = [&](int stage) {
    float* dst = ring + stage * (32 * LDA);
#pragma unroll
    for (int i = 0; i < g::A_VEC_PER_THREAD; ++i) {
      const int id = tid + i * kThreads;
      if (id < 32 * K / 4) {
        if (!areg_trans) {
          const int row = id / (K / 4), c4 = id % (K / 4);
          *reinterpret_cast<float4*>(dst + row * LDA + c4 * 4) = areg[i];
        } else {
          const int m = id >> 3, o = 4 * (id & 7);
          dst[(o + 0) * LDA + m] = areg[i].x;
          dst[(o + 1) * LDA + m] = areg[i].y;
          dst[(o + 2) * LDA + m] = areg[i].z;
          dst[(o + 3) * LDA + m] = areg[i].w;
        }
      }
    }
  };

  if (p.do_grad)
    for (int i = tid; i < g::GACC_FLOATS; i += kThreads) gacc[i] = 0.f;
  tile_fetch_next();
  tile_commit(0);
  if (total_tiles > 1) {
    tile_fetch_next();
    tile_commit(1);
  }
  __syncthreads();

  // running partial sums (per lane)
  float s_l2 = 0.f, s_errz = 0.f, s_wsq = 0.f, s_sur = 0.f;
  float s_va2[NGRP];
#pragma unroll
  for (int i = 0; i < NGRP; ++i) s_va2[i] = 0.f;
  float m_ref = -INFINITY;  // kLossLse: reference of this workgroup's exponentials

  int cur_seg = seg_first;
  int tile = 0;        // tiles consumed so far
  int stage = 0;       // ring stage of the tile being consumed; tile + 2 goes to stage + 2 (mod 3)

  auto flush = [&](int seg) {
    // reduce the per-lane sums and publish this (workgroup, segment) partial
    const int64_t slot = w + seg;
    float vals[kHdrVa2 + NGRP];
    vals[kHdrL2] = s_l2; vals[kHdrErrZ] = s_errz; vals[kHdrWsq] = s_wsq; vals[kHdrSur] = s_sur;
    vals[kHdrMref] = 0.f; vals[5] = 0.f; vals[6] = 0.f; vals[7] = 0.f;
#pragma unroll
    for (int i = 0; i < NGRP; ++i) vals[kHdrVa2 + i] = s_va2[i];
#pragma unroll
    for (int i = 0; i < kHdrVa2 + NGRP; ++i) {
      const float t = wave_sum(vals[i]);
      if (lane == 0) hred[wave * kHdrFloats + i] = t;
    }
    __syncthreads();   // also: every wave has finished its gradient atomics
    if (tid < kHdrVa2 + NGRP) {
      float t = 0.f;
#pragma unroll
      for (int ww = 0; ww < kNW; ++ww) t += hred[ww * kHdrFloats + tid];
      if (tid == kHdrMref) t = m_ref;
      p.slot_hdr[slot * kHdrFloats + tid] = t;
    }
    if (p.do_grad) {
      float* dst = p.slot_grad + slot * int64_t(NBLK * K * K);
      for (int i = tid; i < NBLK * K * K; i += kThreads) {
        const int row = i / K, col = i % K;            // row = blk*K + j
        dst[i] = gacc[row * (K + 1) + col];
        gacc[row * (K + 1) + col] = 0.f;
      }
    }
    __syncthreads();
    s_l2 = s_errz = s_wsq = s_sur = 0.f;
#pragma unroll
    for (int i = 0; i < NGRP; ++i) s_va2[i] = 0.f;
    m_ref = -INFINITY;
  };

  // ---- weights of a strip: B operands, element j(f, h) of the lane's line in wreg[f].
  // Loaded one macro-tile ahead (after the last use of the previous strip's weights).
  float wreg[L / 2];
  auto load_w = [&](int seg, int mis) {
    const int64_t line = int64_t(mis) * kMacroLines + wave * kStripLines + ln;
    const bool valid = line < p.nlines;
    const int64_t ax0 = int64_t(seg) * L;
    if (AXIS == CAFEQ_AXIS_COL) {
      if (p.dtype == CAFEQ_F32) {
        const float* src = static_cast<const float*>(p.W) + line * p.ld + ax0 + 4 * h;
#pragma unroll
        for (int c = 0; c < L / 8; ++c) {
          float4 v = valid ? *reinterpret_cast<const float4*>(src + 8 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
          wreg[4 * c] = v.x; wreg[4 * c + 1] = v.y; wreg[4 * c + 2] = v.z; wreg[4 * c + 3] = v.w;
        }
      } else {
        const uint16_t* src = static_cast<const uint16_t*>(p.W) + line * p.ld + ax0 + 4 * h;
#pragma unroll
        for (int c = 0; c < L / 8; ++c) {
          float4 v = valid ? load4(src + 8 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
          wreg[4 * c] = v.x; wreg[4 * c + 1] = v.y; wreg[4 * c + 2] = v.z; wreg[4 * c + 3] = v.w;
        }
      }
    } else {
      if (p.dtype == CAFEQ_F32) {
        const float* src = static_cast<const float*>(p.W) + (ax0 + 4 * h) * p.ld + line;
#pragma unroll
        for (int f = 0; f < L / 2; ++f)
          wreg[f] = valid ? src[int64_t(8 * (f / 4) + (f % 4)) * p.ld] : 0.f;
      } else {
        const uint16_t* src = static_cast<const uint16_t*>(p.W) + (ax0 + 4 * h) * p.ld + line;
#pragma unroll
        for (int f = 0; f < L / 2; ++f)
          wreg[f] = valid ? bf16_bits_to_f32(src[int64_t(8 * (f / 4) + (f % 4)) * p.ld]) : 0.f;
      }
    }
  };
  load_w(seg_first, mis_first);

#ifdef CAFEQ_CORE_TIMING
  long long tph[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  long long tlast = __builtin_readcyclecounter();
#define CAFEQ_STAMP(i) { const long long tn = __builtin_readcyclecounter(); tph[i] += tn - tlast; tlast = tn; }
#else
#define CAFEQ_STAMP(i)
#endif
  int seg = seg_first, mis = mis_first;
  for (int64_t mt = mt0; mt < mt1; ++mt) {
    CAFEQ_STAMP(0)
    if (seg != cur_seg) {
      if (p.do_inverse || p.do_grad) flush(cur_seg);   // partial buffers exist only for loss calls
      cur_seg = seg;
    }
    const int64_t line = int64_t(mis) * kMacroLines + wave * kStripLines + ln;
    const bool valid = line < p.nlines;
    const int64_t ax0 = int64_t(seg) * L;  // first axis index of the segment
    // the macro-tile after this one
    int nseg_ = seg, nmis = mis + 1;
    if (nmis == mt_per_seg) { nmis = 0; ++nseg_; }

    // ---- forward transform: acc[t] = Afwd tile t (32 x K) times the strip's block
    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bool more = tile + 2 < total_tiles;
      if (more) tile_fetch_next();
      const float* abuf = ring + stage * (32 * LDA) + ln * LDA + 4 * h;
      const int wb = (t / KT) * (K / 2);
      acc[t] = tile_mfma<K>(abuf, [&](int i) { return wreg[wb + i]; });
      if (more) tile_commit(stage == 0 ? 2 : stage - 1);
      __syncthreads();
      ++tile;
      stage = stage == 2 ? 0 : stage + 1;
    }

    CAFEQ_STAMP(1)
    // ---- optional raw output Z
    if (p.Zout && valid) {
      if (AXIS == CAFEQ_AXIS_COL) {
        float* dst = p.Zout + line * p.cols + ax0 + 4 * h;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4*>(dst + 32 * t + 8 * q) =
                make_float4(acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]);
      } else {
        float* dst = p.Zout + (ax0 + 4 * h) * p.cols + line;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) dst[int64_t(32 * t + 8 * (v / 4) + (v % 4)) * p.cols] = acc[t][v];
      }
    }

    CAFEQ_STAMP(2)
    const bool want_q = p.codes || p.scales || p.do_inverse;
    if (want_q) {
      // ---- per-group absmax (+ argmax), codes, error in place
      float gz[NGRP];   // signed value at the arg-max element
      int gj[NGRP];     // its axis index inside the segment
#pragma unroll
      for (int gi = 0; gi < NGRP; ++gi) {
        float a = -1.f, zs = 0.f;
        int j = 0;
#pragma unroll
        for (int f = gi * RPG; f < (gi + 1) * RPG; ++f) {
          const float z = acc[f / 16][f % 16];
          const float v = fabsf(z);
          if (v > a) { a = v; zs = z; j = 8 * (f / 4) + 4 * h + (f % 4); }
        }
        const float oz = __shfl_xor(zs, 32);
        const int oj = __shfl_xor(j, 32);
        const float oa = fabsf(oz);
        if (oa > a || (oa == a && oj < j)) { a = oa; zs = oz; j = oj; }
        gz[gi] = zs; gj[gi] = j;
        const float inv = grid_inv(a, p.grid.qmax);
        const float s = grid_scale(a, p.grid.qmax);
        if (p.scales && valid && h == 0) {
          const int64_t gidx = ax0 / G + gi;   // group index along the axis
          if (AXIS == CAFEQ_AXIS_COL) p.scales[line * (p.cols / G) + gidx] = s;
          else p.scales[gidx * p.cols + line] = s;
        }
#pragma unroll
        for (int f4 = gi * RPG / 4; f4 < (gi + 1) * RPG / 4; ++f4) {
          float q[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int f = 4 * f4 + e;
            const float z = acc[f / 16][f % 16];
            q[e] = grid_code(z, inv, p.grid);
            const float er = __fmul_rn(q[e], s) - z;
            s_errz = fmaf(er, er, s_errz);
            acc[f / 16][f % 16] = er;
          }
          if (p.codes && valid) {
            const int j0 = 8 * f4 + 4 * h;
            if (AXIS == CAFEQ_AXIS_COL) {
              *reinterpret_cast<uint32_t*>(p.codes + line * p.cols + ax0 + j0) = pack4(q[0], q[1], q[2], q[3]);
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e) p.codes[(ax0 + j0 + e) * p.cols + line] = int8_t(int(q[e]));
            }
          }
        }
        if (p.do_inverse) {
          const float a2 = a * a;
          if (h == 0) s_va2[gi] += a2;
          if (p.loss_kind == kLossSur && h == 0) s_sur = fmaf(a2, p.rG[seg * NGRP + gi], s_sur);
        }
      }

      if (p.do_inverse) {
#pragma unroll
        for (int f = 0; f < L / 2; ++f) s_wsq = fmaf(wreg[f], wreg[f], s_wsq);
      }

      // ---- LogSumExp bookkeeping: exponentials relative to a workgroup-wide running reference
      const bool lse_on = p.loss_kind == kLossLse && p.do_inverse;
      if (lse_on) {
        float mx = 0.f;
#pragma unroll
        for (int gi = 0; gi < NGRP; ++gi) mx = fmaxf(mx, valid ? fabsf(gz[gi]) : 0.f);
        mx = cluster_allmax<64>(mx);
        if (lane == 0) wmax[wave] = mx;
        __syncthreads();
        float nm = wmax[0];
#pragma unroll
        for (int ww = 1; ww < kNW; ++ww) nm = fmaxf(nm, wmax[ww]);
        if (nm > m_ref) {                                       // uniform over the workgroup
          const float sc = __expf(p.lse_t * (m_ref - nm));      // 0 on the first macro-tile
          if (p.do_grad)
            for (int i = tid; i < NBLK * K * (K + 1); i += kThreads) gacc[i] *= sc;
          s_sur *= sc;
          m_ref = nm;
        }
        __syncthreads();
      }

      // ---- gradient of the surrogate through Z: rank-1 updates into the LDS accumulator
      if (p.do_grad || lse_on) {
#pragma unroll
        for (int gi = 0; gi < NGRP; ++gi) {
          float coef;
          if (p.loss_kind == kLossSur) {
            coef = 2.f * p.beta * p.rG[seg * NGRP + gi] * gz[gi];
          } else {
            const float e = valid ? __expf(p.lse_t * (fabsf(gz[gi]) - m_ref)) : 0.f;
            if (h == 0) s_sur += e;
            coef = gz[gi] < 0.f ? -e : e;
          }
          if (!p.do_grad) continue;
          // blocks this group can touch
          constexpr int BPG = G > K ? G / K : 1;
          const int blk0 = (gi * G) / K;
#pragma unroll
          for (int bb = 0; bb < BPG; ++bb) {
            const int blk = blk0 + bb;
            const int jl = gj[gi] - blk * K;
            if (jl >= 0 && jl < K && coef != 0.f) {
              float* row = gacc + (blk * K + jl) * (K + 1) + 4 * h;
#pragma unroll
              for (int r = 0; r < K / 2; ++r)
                atomicAdd(row + 8 * (r / 4) + (r % 4), coef * wreg[blk * (K / 2) + r]);
            }
          }
        }
      }
    }

    CAFEQ_STAMP(3)
    // ---- the next strip's weights: wreg is dead from here on, the loads land during the
    // inverse phase
    if (mt + 1 < mt1) load_w(nseg_, nmis);

    CAFEQ_STAMP(4)
    // ---- inverse transform of the error and the l2 proxy
    if (p.do_inverse) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bool more = tile + 2 < total_tiles;
        if (more) tile_fetch_next();
        const float* abuf = ring + stage * (32 * LDA) + ln * LDA + 4 * h;
        const int eb = (t / KT) * (K / 2);   // first error register of this tile's block
        const floatx16 d = tile_mfma<K>(abuf, [&](int i) { return acc[(eb + i) / 16][(eb + i) % 16]; });
#pragma unroll
        for (int v = 0; v < 16; ++v) s_l2 = fmaf(d[v], d[v], s_l2);
        if (more) tile_commit(stage == 0 ? 2 : stage - 1);
        __syncthreads();
        ++tile;
        stage = stage == 2 ? 0 : stage + 1;
      }
    }
    CAFEQ_STAMP(5)
    seg = nseg_;
    mis = nmis;
  }
  if (p.do_inverse || p.do_grad) flush(cur_seg);
#ifdef CAFEQ_CORE_TIMING
  CAFEQ_STAMP(6)
  if (p.dbg && lane == 0 && wave == 0)
    for (int i = 0; i < 8; ++i) p.dbg[blockIdx.x * 8 + i] = tph[i];
#endif
}

}  // namespace cafeq
