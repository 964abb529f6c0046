// Gradient pass over prepared weights for 128 x 128 transform blocks: gradT_b += W_b^T S_b (columns) /
// S_b W_b^T (rows), S holding one non-zero per (line, group) at the group's arg-max (paper Sec. 4.1: gradient
// of the surrogate through the transformed weights; Sec. 4.2: of the LogSumExp surrogate).
//
// The weights do not change over a learning run, so cafeq_prepare_weights also stores them in the form THIS
// contraction consumes -- it runs over the lines, so the matrix instruction wants, per input, eight consecutive
// lines side by side, i.e. the transpose of what the loss pass reads.  Per tile of 128 lines x 128 inputs:
//   [step of 16 lines: 8][tile of 32 inputs: 4][part: hi, mid][lane: 64][16 bytes]
// with lane = input % 32 + 32 * (line / 8 % 2) holding the bfloat16 parts of lines 8 (line / 8) .. + 7: one
// contiguous kilobyte per operand of v_mfma_f32_32x32x16_bf16, so a wave loads its operands from memory
// straight into registers (no float32 split, no transposition through LDS in the hot loop).
//
// A workgroup (four waves) owns a contiguous, block-major range of such tiles.  Wave m accumulates the four
// 32 x 32 tiles of all 128 output rows and inputs 32 m .. + 31: its W operands are private to it (every byte
// of the weights is requested once), held a whole tile ahead -- each of the eight steps has its own registers,
// refilled with the next tile's step as soon as it has been used, so a wave keeps 16 KB in flight; the S
// operands are shared through LDS, where they sit in operand order too: the area is zeroed once, per tile every
// lane drops its line's coefficient parts (two bytes each) where the line's arg-max falls, and takes them out
// again afterwards.  Three part products (S lo x W hi, S hi x W mid, S hi x W hi), float32 accumulation; one partial per
// (workgroup, block) in the layout of the generic gradient pass, reduced in fixed order by reduce_grad_kernel.
#include <atomic>

#include "cafeq_internal.hpp"
#include "xform_core.hpp"
#include "loss_reduce.hpp"

namespace cafeq {
namespace {

constexpr int kGvLines = 128;                     // lines of a tile
constexpr int kGvOperandB = 1024;                 // one matrix-instruction operand
constexpr int kGvSbufB = 4 * 8 * 2 * kGvOperandB; // S operands of a tile: [tile row 4][step 8][part 2]
constexpr int kGvLds = kGvSbufB + 64;

__global__ __launch_bounds__(kThreads, 2) void grad_v2_kernel(const CoreParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sbuf = smem;
  float* red = reinterpret_cast<float*>(smem + kGvSbufB);   // [kNW]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5;

  int64_t w = blockIdx.x;
  if ((p.nwg & 7) == 0) w = int64_t(blockIdx.x & 7) * (p.nwg >> 3) + (blockIdx.x >> 3);
  const int64_t mt0 = chunk_begin(w, p.n_mt, p.nwg), mt1 = chunk_begin(w + 1, p.n_mt, p.nwg);

  for (int i = tid; i < kGvSbufB / 16; i += kThreads) reinterpret_cast<uint4*>(sbuf)[i] = make_uint4(0u, 0u, 0u, 0u);

  // kLossLse: exponentials relative to the member's largest group maximum
  float m_mem = 0.f;
  if (p.loss_kind == kLossLse) {
    float m = -INFINITY;
    for (int i = tid; i < p.nslot_ref; i += kThreads) m = fmaxf(m, p.hdr_ref[int64_t(i) * kHdrFloats + kHdrMref]);
    m = cluster_allmax<64>(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m_mem = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    if (blockIdx.x == 0 && tid == 0) *p.member_ref = m_mem;
  }
  __syncthreads();
  if (mt0 >= mt1) return;

  const int mt_per_seg = int(p.mt_per_seg);
  int seg = int(mt0 / p.mt_per_seg);                  // block of 128 inputs
  int mis = int(mt0 - int64_t(seg) * p.mt_per_seg);
  int cur_seg = seg;

  // gt[i]: output rows 32 i .. + 31, inputs 32 wave .. + 31; element [8 (v / 4) + 4 h + v % 4][ln] of the tile
  floatx16 gt[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) gt[i][v] = 0.f;

  // (uniform row pointers + one 32-bit lane offset: no per-store address registers to keep across the loop)
  const uint32_t floff = uint32_t(4 * h * 128 + wave * 32 + ln);
  auto flush = [&](int sg_) {
    float* dst = p.slot_grad + (w + sg_) * int64_t(128 * 128);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float* rowp = dst + (i * 32 + 8 * (v / 4) + (v % 4)) * 128;
        rowp[floff] = gt[i][v];
        gt[i][v] = 0.f;
      }
  };

  // ---- the S side: this lane stages line L = 32 wave + ln of the tile for the tile rows 2 h and 2 h + 1
  const int L = wave * 32 + ln;
  const int sl_off = ((L >> 4) * 2) * kGvOperandB + ((L >> 3) & 1) * 32 * 16 + (L & 7) * 2;   // step, lane half, slot
  // the rows' groups change with the block only: group index, first output of the row inside its group, and
  // (surrogate) the group's sum of rho
  int64_t gidx[2];
  int joff[2];
  float rgv[2];
  auto row_groups = [&](int sg_) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t aj = int64_t(sg_) * 128 + 32 * (2 * h + i);
      gidx[i] = aj / p.grp;
      joff[i] = int(aj - gidx[i] * p.grp);
      rgv[i] = p.loss_kind == kLossSur ? p.rG[gidx[i]] : 0.f;
    }
  };
  // (loads without branches: lines past the matrix read the last line's record and are masked when used, so
  // that the wait for these values never has to cover the operand loads issued after them)
  float2 recv[2];
  bool rvalid = false;
  auto load_rec = [&](int ms_) {
    const int64_t line = int64_t(ms_) * kGvLines + L;
    rvalid = line < p.nlines;
    const int64_t lc = rvalid ? line : p.nlines - 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) recv[i] = p.rec[gidx[i] * p.nlines + lc];
  };
  int woff[2] = {-1, -1};   // where this lane's coefficients sit in the S area (-1: nowhere)

  // ---- the W side: the operands of the wave's input tile, one register set per step of a tile
  const unsigned char* gbase = p.prep_gtiles + wave * 2 * kGvOperandB + lane * 16;
  auto tile_ptr = [&](int sg_, int ms_) { return gbase + (int64_t(sg_) * mt_per_seg + ms_) * int64_t(8 * 4 * 2 * kGvOperandB); };
  uintx4 breg[8][2];   // [step][part]
  auto load_step = [&](const unsigned char* tp, int s) {
#pragma unroll
    for (int part = 0; part < 2; ++part)
      breg[s][part] = *reinterpret_cast<const uintx4*>(tp + (s * 4 * 2 + part) * kGvOperandB);
  };

  const unsigned char* tile = tile_ptr(seg, mis);
  row_groups(seg);
  load_rec(mis);   // (before the operand loads, and these in the order of their use, as in the loop: the waits
                   // the compiler places in the loop cover both ways into it)
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    load_step(tile, s);
    __builtin_amdgcn_sched_barrier(0);
  }

  for (int64_t mt = mt0; mt < mt1; ++mt) {
    if (seg != cur_seg) {
      flush(cur_seg);
      cur_seg = seg;
    }
    int nseg_ = seg, nmis = mis + 1;
    if (nmis == mt_per_seg) { nmis = 0; ++nseg_; }
    const bool has_next = mt + 1 < mt1;
    // (past the range's end the prefetches re-read this tile: always in bounds, never used)
    const unsigned char* ntile = has_next ? tile_ptr(nseg_, nmis) : tile;

    // ---- this tile's S entries: out with the previous tile's, in with the new ones
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (woff[i] >= 0) {
        *reinterpret_cast<uint16_t*>(sbuf + woff[i]) = 0;
        *reinterpret_cast<uint16_t*>(sbuf + woff[i] + kGvOperandB) = 0;
        woff[i] = -1;
      }
      const float2 rc = recv[i];
      const int jj = __float_as_int(rc.y) - joff[i];
      if (rvalid && jj >= 0 && jj < 32) {
        float coef;
        if (p.loss_kind == kLossSur) {
          coef = 2.f * p.beta * rgv[i] * rc.x;
        } else {
          const float e = __expf(p.lse_t * (fabsf(rc.x) - m_mem));
          coef = rc.x < 0.f ? -e : e;
        }
        // coefficient as an exact-to-16-bit bfloat16 pair
        const uint32_t ch = pack_bf16(coef, 0.f);
        const uint32_t cl = pack_bf16(coef - bf16_lo_f32(ch), 0.f);
        const int off = (2 * h + i) * 8 * 2 * kGvOperandB + sl_off + jj * 16;
        *reinterpret_cast<uint16_t*>(sbuf + off) = uint16_t(ch);
        *reinterpret_cast<uint16_t*>(sbuf + off + kGvOperandB) = uint16_t(cl);
        woff[i] = off;
      }
    }
    // the next tile's records (past the range's end: this tile's again, never used)
    if (has_next && nseg_ != seg) row_groups(nseg_);
    load_rec(has_next ? nmis : mis);
    __syncthreads();

    // ---- G[j][m] += sum over the tile's lines of S[line][j] * W[line][m], 16 lines per step: three part
    // products (S lo x W hi, S hi x W mid, S hi x W hi), each over the four tile rows, so that consecutive MFMAs
    // never wait on each other's accumulator.  The S lo operands of the next step are requested as soon as the
    // first product has issued, the S hi ones after the last, and the step's W registers are refilled with the
    // next tile's; the scheduling fences keep the compiler from moving the requests to their uses.
    bf16x8 ash[4], asl[4];   // [tile row]
    auto read_s = [&](bf16x8 (&dst)[4], int s, int part) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        dst[i] = as_bf16x8(*reinterpret_cast<const uintx4*>(sbuf + ((i * 8 + s) * 2 + part) * kGvOperandB + lane * 16));
    };
    read_s(asl, 0, 1);
    read_s(ash, 0, 0);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 bh = as_bf16x8(breg[s][0]), bm = as_bf16x8(breg[s][1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) gt[i] = CAFEQ_MFMA_BF16(asl[i], bh, gt[i]);
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < 8) read_s(asl, s + 1, 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) gt[i] = CAFEQ_MFMA_BF16(ash[i], bm, gt[i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) gt[i] = CAFEQ_MFMA_BF16(ash[i], bh, gt[i]);
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < 8) read_s(ash, s + 1, 0);
      load_step(ntile, s);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();   // the S area is rewritten for the next tile
    tile = ntile;
    seg = nseg_;
    mis = nmis;
  }
  flush(cur_seg);
}

// The same contraction with one workgroup per (matrix, block): eight waves, the first four take the block's even
// tiles and the last four the odd ones (an S area each), the two halves' accumulators are added through LDS at
// the end and the block's gradient is written in its final form -- no partials, no reduction pass.  For calls
// whose blocks fill the chip once (the pair on the 9B-shaped MLP: 2 x 112 blocks on 256 compute units) and
// whose groups' coefficients are final when the pass starts: the surrogate's 2 beta rho_G z, or the LogSumExp's
// exp(t (|z| - m*)) / S with the pair's m* and S already reduced (lse_ms).
struct GvMember {
  const unsigned char* gtiles;
  const float2* rec;
  const float* rG;
  float* out;            // [nseg][128][128]
  int64_t nlines;
  int mt_per_seg, nseg, grp, transpose_out;
};
struct GvOwnerArgs {
  GvMember m[2];
  int nmem, loss_kind;
  float beta, lse_t;
  const double* lse_ms;   // kLossLse: {m*, S}, unless fold is set
  // fold != 0: the call's loss reduction runs inside this launch instead of before it -- every workgroup forms
  // {m*, S} from the partial headers itself (kLossLse), workgroup 0 also writes the losses
  int fold;
  LossArgs la;
};

__global__ __launch_bounds__(512, 1) void grad_v2_owner_kernel(const GvOwnerArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5;
  const int half = wave >> 2, wq = wave & 3;
  unsigned char* sbuf = smem + half * kGvSbufB;

  const int mi = (a.nmem > 1 && int(blockIdx.x) >= a.m[0].nseg) ? 1 : 0;
  const GvMember& M = a.m[mi];
  const int seg = int(blockIdx.x) - (mi ? a.m[0].nseg : 0);
  const int mt_per_seg = M.mt_per_seg;
  const int niter = (mt_per_seg + 1) / 2;

  for (int i = tid; i < 2 * kGvSbufB / 16; i += 512) reinterpret_cast<uint4*>(smem)[i] = make_uint4(0u, 0u, 0u, 0u);
  float mstar = 0.f, inv_s = 1.f;
  if (a.loss_kind == kLossLse && !a.fold) {
    mstar = float(a.lse_ms[0]);
    inv_s = float(1.0 / a.lse_ms[1]);
  }
  __syncthreads();

  floatx16 gt[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) gt[i][v] = 0.f;

  // ---- the S side (as in grad_v2_kernel; the rows' groups are fixed: one block per workgroup)
  const int L = wq * 32 + ln;
  const int sl_off = ((L >> 4) * 2) * kGvOperandB + ((L >> 3) & 1) * 32 * 16 + (L & 7) * 2;
  int64_t gidx[2];
  int joff[2];
  float rgv[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int64_t aj = int64_t(seg) * 128 + 32 * (2 * h + i);
    gidx[i] = aj / M.grp;
    joff[i] = int(aj - gidx[i] * M.grp);
    rgv[i] = a.loss_kind == kLossSur ? M.rG[gidx[i]] : 0.f;
  }
  float2 recv[2];
  bool rvalid = false;
  auto load_rec = [&](int ms_) {
    const int64_t line = int64_t(ms_) * kGvLines + L;
    rvalid = line < M.nlines;
    const int64_t lc = rvalid ? line : M.nlines - 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) recv[i] = M.rec[gidx[i] * M.nlines + lc];
  };
  int woff[2] = {-1, -1};

  // ---- the W side
  const unsigned char* gbase = M.gtiles + wq * 2 * kGvOperandB + lane * 16;
  auto tile_ptr = [&](int ms_) { return gbase + (int64_t(seg) * mt_per_seg + ms_) * int64_t(8 * 4 * 2 * kGvOperandB); };
  uintx4 breg[8][2];
  auto load_step = [&](const unsigned char* tp, int s) {
#pragma unroll
    for (int part = 0; part < 2; ++part)
      breg[s][part] = *reinterpret_cast<const uintx4*>(tp + (s * 4 * 2 + part) * kGvOperandB);
  };
  // (a half without a tile of its own -- the odd half of a block with one tile -- reads tile 0 and skips the work)
  int mis = half < mt_per_seg ? half : 0;
  const unsigned char* tile = tile_ptr(mis);
  load_rec(mis);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    load_step(tile, s);
    __builtin_amdgcn_sched_barrier(0);
  }

  if (a.fold) {
    // (after the first tile's requests, which are in flight meanwhile)
    double* red = reinterpret_cast<double*>(smem + 2 * kGvSbufB);
    if (a.loss_kind == kLossLse) {
      double m = 0, sm = 1;
      reduce_losses_body<512>(a.la, red, blockIdx.x == 0, &m, &sm);
      mstar = float(m);
      inv_s = float(1.0 / sm);
    } else if (blockIdx.x == 0) {
      double m, sm;
      reduce_losses_body<512>(a.la, red, true, &m, &sm);
    }
  }

  for (int it = 0; it < niter; ++it) {
    const bool active = 2 * it + half < mt_per_seg;          // uniform over the wave
    const bool has_next = 2 * (it + 1) + half < mt_per_seg;
    const int nmis = has_next ? mis + 2 : mis;
    const unsigned char* ntile = tile_ptr(nmis);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (woff[i] >= 0) {
        *reinterpret_cast<uint16_t*>(sbuf + woff[i]) = 0;
        *reinterpret_cast<uint16_t*>(sbuf + woff[i] + kGvOperandB) = 0;
        woff[i] = -1;
      }
      const float2 rc = recv[i];
      const int jj = __float_as_int(rc.y) - joff[i];
      if (active && rvalid && jj >= 0 && jj < 32) {
        float coef;
        if (a.loss_kind == kLossSur) {
          coef = 2.f * a.beta * rgv[i] * rc.x;
        } else {
          const float e = __expf(a.lse_t * (fabsf(rc.x) - mstar)) * inv_s;
          coef = rc.x < 0.f ? -e : e;
        }
        const uint32_t ch = pack_bf16(coef, 0.f);
        const uint32_t cl = pack_bf16(coef - bf16_lo_f32(ch), 0.f);
        const int off = (2 * h + i) * 8 * 2 * kGvOperandB + sl_off + jj * 16;
        *reinterpret_cast<uint16_t*>(sbuf + off) = uint16_t(ch);
        *reinterpret_cast<uint16_t*>(sbuf + off + kGvOperandB) = uint16_t(cl);
        woff[i] = off;
      }
    }
    load_rec(nmis);
    __syncthreads();

    bf16x8 ash[4], asl[4];
    auto read_s = [&](bf16x8 (&dst)[4], int s, int part) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        dst[i] = as_bf16x8(*reinterpret_cast<const uintx4*>(sbuf + ((i * 8 + s) * 2 + part) * kGvOperandB + lane * 16));
    };
    read_s(asl, 0, 1);
    read_s(ash, 0, 0);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 bh = as_bf16x8(breg[s][0]), bm = as_bf16x8(breg[s][1]);
      __builtin_amdgcn_sched_barrier(0);
      // (an inactive half multiplies zeros: its S area is empty)
#pragma unroll
      for (int i = 0; i < 4; ++i) gt[i] = CAFEQ_MFMA_BF16(asl[i], bh, gt[i]);
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < 8) read_s(asl, s + 1, 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) gt[i] = CAFEQ_MFMA_BF16(ash[i], bm, gt[i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) gt[i] = CAFEQ_MFMA_BF16(ash[i], bh, gt[i]);
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < 8) read_s(ash, s + 1, 0);
      load_step(ntile, s);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    tile = ntile;
    mis = nmis;
  }

  // ---- the two halves' sums, and out: element [j = 32 i + 8 (v / 4) + 4 h + v % 4][m = 32 wq + ln]
  float* xb = reinterpret_cast<float*>(smem);   // [wq][i][v][lane]: 64 KB (the S areas are done with)
  if (half == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) xb[((wq * 4 + i) * 16 + v) * 64 + lane] = gt[i][v];
  }
  __syncthreads();
  if (half == 0) {
    float* dst = M.out + int64_t(seg) * (128 * 128);
    const uint32_t lo_n = uint32_t(4 * h * 128 + wq * 32 + ln);          // [j][m]
    const uint32_t lo_t = uint32_t((wq * 32 + ln) * 128 + 4 * h);        // [m][j]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float g = gt[i][v] + xb[((wq * 4 + i) * 16 + v) * 64 + lane];
        const int jc = i * 32 + 8 * (v / 4) + (v % 4);                   // j without the lane-half term
        if (M.transpose_out) (dst + jc)[lo_t] = g;
        else (dst + jc * 128)[lo_n] = g;
      }
  }
}

// One workgroup per tile of 128 lines x 128 inputs: the bfloat16 hi + mid parts of every weight (hi = the
// round-to-nearest of the value, mid = that of the remainder: 16 significant bits), in operand order.
struct GtileArgs {
  const void* W; int dtype; int64_t ld; int axis;
  int64_t nlines, nmt;
  unsigned char* gtiles;
};
__global__ __launch_bounds__(256) void prepare_gtiles_kernel(const GtileArgs a) {
  const int64_t tix = blockIdx.x;
  const int64_t seg = tix / a.nmt, mis = tix - seg * a.nmt;
  unsigned char* tp = a.gtiles + tix * int64_t(8 * 4 * 2 * kGvOperandB);
  for (int s = 0; s < 8; ++s) {
    const int lane = threadIdx.x & 63, mt = threadIdx.x >> 6;
    const int ln = lane & 31, h = lane >> 5;
    const int64_t ax = seg * 128 + 32 * mt + ln, line0 = mis * kGvLines + 16 * s + 8 * h;
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t line = line0 + e;
      x[e] = 0.f;
      if (line < a.nlines) {
        const int64_t off = a.axis == CAFEQ_AXIS_COL ? line * a.ld + ax : ax * a.ld + line;
        x[e] = a.dtype == CAFEQ_F32 ? static_cast<const float*>(a.W)[off]
                                    : bf16_bits_to_f32(static_cast<const uint16_t*>(a.W)[off]);
      }
    }
    uint32_t hi[4], mid[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      hi[e2] = pack_bf16(x[2 * e2], x[2 * e2 + 1]);
      mid[e2] = pack_bf16(x[2 * e2] - bf16_lo_f32(hi[e2]), x[2 * e2 + 1] - bf16_hi_f32(hi[e2]));
    }
    unsigned char* op = tp + ((s * 4 + mt) * 2) * kGvOperandB + lane * 16;
    *reinterpret_cast<uint4*>(op) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    *reinterpret_cast<uint4*>(op + kGvOperandB) = make_uint4(mid[0], mid[1], mid[2], mid[3]);
  }
}

}  // namespace

size_t prepared_gtiles_bytes(int64_t nlines, int64_t naxis) {
  const int64_t nmt = (nlines + kGvLines - 1) / kGvLines;
  return size_t(nmt) * size_t(naxis / 128) * size_t(8 * 4 * 2 * kGvOperandB);
}

int launch_prepare_gtiles(const cafeq_mat* W, int axis, unsigned char* gtiles, hipStream_t st) {
  const bool col = axis == CAFEQ_AXIS_COL;
  const int64_t nlines = col ? W->rows : W->cols, naxis = col ? W->cols : W->rows;
  if (naxis % 128 != 0) return CAFEQ_ERR_BAD_SHAPE;
  GtileArgs a;
  a.W = W->data; a.dtype = W->dtype; a.ld = W->ld; a.axis = axis;
  a.nlines = nlines; a.nmt = (nlines + kGvLines - 1) / kGvLines;
  a.gtiles = gtiles;
  hipLaunchKernelGGL(prepare_gtiles_kernel, dim3(unsigned(a.nmt * (naxis / 128))), dim3(256), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

// Both members of a pair (or one matrix) with one workgroup per block; see grad_v2_owner_kernel.
int launch_grad_v2_owner(const GradOwnerJob* jobs, int n, int loss_kind, float beta, float lse_t, const double* lse_ms,
                         hipStream_t st, const LossArgs* fold) {
  if (n < 1 || n > 2) return CAFEQ_ERR_INVALID_ARG;
  GvOwnerArgs a;
  int nwg = 0;
  for (int i = 0; i < n; ++i) {
    const GradOwnerJob& j = jobs[i];
    if (!j.gtiles || !j.rec || !j.out || j.grp < 32 || j.grp % 32 != 0 || j.nseg < 1) return CAFEQ_ERR_INVALID_ARG;
    if (loss_kind == kLossSur && !j.rG) return CAFEQ_ERR_INVALID_ARG;
    a.m[i].gtiles = j.gtiles; a.m[i].rec = j.rec; a.m[i].rG = j.rG; a.m[i].out = j.out;
    a.m[i].nlines = j.nlines; a.m[i].mt_per_seg = int((j.nlines + kGvLines - 1) / kGvLines);
    a.m[i].nseg = j.nseg; a.m[i].grp = j.grp; a.m[i].transpose_out = j.transpose_out;
    nwg += j.nseg;
  }
  if (n == 1) a.m[1] = a.m[0];
  if (loss_kind == kLossLse && !lse_ms) return CAFEQ_ERR_INVALID_ARG;
  a.nmem = n; a.loss_kind = loss_kind; a.beta = beta; a.lse_t = lse_t; a.lse_ms = lse_ms;
  a.fold = fold ? 1 : 0;
  if (fold) {
    if (fold->kind != loss_kind || !fold->hdrA || !fold->losses || (loss_kind == kLossLse && !fold->lse_ms))
      return CAFEQ_ERR_INVALID_ARG;
    a.la = *fold;
  } else {
    a.la = LossArgs{};
  }
  static std::atomic<bool> attr_set{false};
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(grad_v2_owner_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return CAFEQ_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL(grad_v2_owner_kernel, dim3(unsigned(nwg)), dim3(512), 2 * kGvSbufB + 5 * 8 * sizeof(double), st, a);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_grad_v2(const CoreParams& p, hipStream_t st) {
  if (!p.prep_gtiles || !p.rec || !p.slot_grad || p.grp < 32 || p.grp % 32 != 0) return CAFEQ_ERR_INVALID_ARG;
  if (p.mt_per_seg != (p.nlines + kGvLines - 1) / kGvLines) return CAFEQ_ERR_INVALID_ARG;
  static std::atomic<bool> attr_set{false};
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(grad_v2_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return CAFEQ_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL(grad_v2_kernel, dim3(unsigned(p.nwg)), dim3(kThreads), kGvLds, st, p);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

}  // namespace cafeq
