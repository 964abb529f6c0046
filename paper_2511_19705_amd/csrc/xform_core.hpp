// Fused block-transform / quantize / inverse-transform / loss / gradient kernel (gfx950).
//
// Work decomposition.  A "line" is one vector along the transformed axis (a row of W for
// AXIS_COL, a column for AXIS_ROW).  The axis is cut into segments of L = max(K, G)
// elements (K: transform block, G: quantization group), so a segment holds whole blocks
// and whole groups.  One wavefront owns a strip of 32 lines x one segment and computes
//   Z^T[j][line] = sum_m Afwd[j][m] * W[line][m]
// on the matrix cores with the transform tile as the A operand (from LDS) and the weights as
// the B operand, read from global memory straight into the lane that consumes them.  In the
// 32x32 accumulator layout a lane then holds, for ONE line, the axis indices
//   j(f, h) = 8*(f/4) + 4*h + f%4,   f = 0..L/2-1,  h = lane/32,
// so a group's absmax is a scan over registers plus one exchange with lane^32, the
// quantization error E replaces Z in the same registers, and -- because registers 8c..8c+7
// of lane (line, h) are exactly the eight inputs 16c + 8u + 4h + e (u < 2, e < 4) that this
// lane feeds to MFMA step c -- those registers are the B operand of the inverse transform
// D^T = Ainv * E^T without any data movement.  Z, E and D never leave the register file; W
// is read from memory once.
//
// Arithmetic.  There is no fast fp32 matrix path on this part (157 TFLOP/s against
// 2.5 PFLOP/s for 16-bit operands), so every fp32 operand x is split exactly into bfloat16
// parts x = hi + mid + lo (8 mantissa bits each) and the products are formed with
// v_mfma_f32_32x32x16_bf16, accumulating in fp32:
//   forward  : 6 products (hi.hi, hi.mid, mid.hi, mid.mid, hi.lo, lo.hi) -- the dropped terms are
//              below 2^-24 relative, so Z is as accurate as an fp32 FMA chain (measured: slightly
//              better than the fp32 MFMA), which the tie-exact code comparison needs;
//   inverse  : 3 products (hi.hi, hi.mid, mid.hi), relative error ~5e-6 per element of D, ample for
//              the 1e-4 budget of the l2 proxy;
//   gradient : d/dZ is sparse (one non-zero per group, at the arg-max).  G[j][m] = sum_lines
//              S[line][j] W[line][m] contracts over LINES, which live in lanes; the strip's W parts
//              (hi, mid) are therefore staged through LDS transposed ([m][line]) and each wave
//              accumulates its share of the k x k tiles in registers with 3 products per step.
// Products of bfloat16 pairs are exact in fp32, so the only roundings are the accumulations.
// The gradient-free variant over 128 x 128 blocks (F16 below) runs the forward contraction on TWO
// float16 parts per operand instead (11 significant bits each; three products hi.hi, hi.lo, lo.hi;
// power-of-two scaling per line and per block keeps the parts inside float16's exponent range).
//
// The transform tiles (32 outputs x K inputs, pre-split into bf16 planes by a preparation
// kernel, columns permuted so that a lane's eight inputs are one 128-bit LDS read) stream
// through an LDS ring shared by the workgroup's waves, fetched two tile-steps ahead from L2;
// one barrier per tile step.  Workgroups are persistent: each takes a contiguous range of
// macro-tiles (segment-major), keeps loss partial sums and the gradient tiles in registers and
// writes one partial per (workgroup, segment) that a finishing kernel reduces in fixed order.
#pragma once
#include "cafeq_internal.hpp"

namespace cafeq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kNW = 4;              // waves per workgroup
constexpr int kThreads = kNW * 64;  // threads per workgroup
constexpr int kStripLines = 32;     // lines per wave
constexpr int kMacroLines = kNW * kStripLines;
constexpr int kFwdPlanes = 3, kInvPlanes = 2;

__host__ __device__ constexpr int cmax(int a, int b) { return a > b ? a : b; }

// header layout of one partial (floats)
constexpr int kHdrL2 = 0, kHdrErrZ = 1, kHdrWsq = 2, kHdrSur = 3, kHdrMref = 4, kHdrVa2 = 8;
constexpr int kHdrFloats = 8 + 32;  // up to 32 groups per segment

template <int K, int G>
struct Geo {
  static constexpr int L = cmax(K, G);
  static constexpr int NBLK = L / K;      // transform blocks per segment
  static constexpr int NT = L / 32;       // 32-output tiles per segment
  static constexpr int KT = K / 32;       // tiles per block
  static constexpr int NGRP = L / G;      // groups per segment
  static constexpr int RPG = G / 2;       // accumulator registers per group per lane
  // A ring stage holds the operand slab of 32 consecutive inputs of one block: all K output
  // rows, 64 bytes per row (four 16-byte chunks: MFMA step 2s+c2, lane half h -> chunk 2*c2+h,
  // stored at chunk ^ ((row >> 2) & 3) so that 16 lanes reading one chunk hit 64 distinct banks)
  static constexpr int PLANEB = K * 64;                    // one plane of one stage
  static constexpr int STAGEB = kFwdPlanes * PLANEB;       // one ring stage
  static constexpr int RING_STAGES = (L == 32 || K > 128) ? 2 : 3;   // fetch distance RING_STAGES - 1 <= NT
  static constexpr int RINGB = RING_STAGES * STAGEB;
  // gradient staging: W parts (hi, mid) transposed [m][line], per-group arg-max / coefficient
  static constexpr int WST_ROWB = 2 * kMacroLines + 16;
  static constexpr int WST_PLANEB = L * WST_ROWB;
  static constexpr int GRADB = 2 * WST_PLANEB + NGRP * kMacroLines * (2 + 4);
  static constexpr int GT_ROWS = (NT + kNW - 1) / kNW;     // tile rows of the gradient per wave
  static constexpr int GT = GT_ROWS * KT;                  // gradient tiles per wave
  static constexpr int A_VEC_PER_THREAD = (STAGEB / 16 + kThreads - 1) / kThreads;
  static constexpr int MISCB = (kNW * kHdrFloats + kNW + 4) * 4;
  // the gradient needs its staging area next to the ring in the 160 KB of LDS and at most
  // eight accumulator tiles per wave
  static constexpr bool GRAD_OK = RINGB + GRADB + MISCB <= 160 * 1024 && GT <= 8;
  static constexpr int GT_ALLOC = GRAD_OK ? GT : 1;
};

enum : int { kLossSur = 0, kLossLse = 1 };

struct CoreParams {
  const void* W;
  int dtype;
  int64_t rows, cols, ld;
  const uint16_t* Afwd;  // [nb][K/32 stages][3 planes][K][32] bf16: forward operand in ring-stage order
  const uint16_t* Ainv;  // [nb][K/32 stages][2 planes][K][32] bf16: inverse operand
  const float* fscale;   // half-precision forward (F16 variant; else null): Afwd holds two float16 planes per stage of
                         // the block scaled by a power of two, fscale[block] is the factor that undoes that scale
  int rep;               // AXIS_ROW: row-block q uses block q / rep
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
  // two-pass gradient: the gradient-free pass records, per (group, line), the signed value at the
  // group's arg-max and its axis index inside the segment; the gradient pass reads them back
  float2* rec;              // [nseg * NGRP][nlines]: (value, index as int bits); may be null
  const float* hdr_ref;     // gradient pass, kLossLse: the first pass's partial headers ...
  int nslot_ref;            // ... and their number: the member's reference is their largest m_ref
  float* member_ref;        // gradient pass, kLossLse: [1] receives that reference
  // Groups longer than a segment (a whole channel, or any multiple of the segment): gspan = segments per
  // group.  A first, forward-only sweep records every segment's arg-max (rec), a small kernel combines the
  // records of a group's segments into grec[group][line] = (signed value at the group's arg-max, its index
  // inside the group), and the loss sweep takes the group's absmax from there instead of its own scan.
  int longg;                // run the long-group kernel variant (both of its sweeps)
  int gspan;                // 1: every group lies inside one segment
  const float2* grec;       // loss sweep with gspan > 1 (else null)
  // gradient pass: group length along the axis, records indexed [axis group][line], index inside the group
  int grp;
  // loss pass over prepared weights (loss_v2.hip): tiles of two float16 parts, per-line factors, ||W||^2
  const unsigned char* prep_planes;
  const float* prep_lscale;
  const float* prep_wsq;
  const float* fscale_inv;  // per-block factor of the float16 inverse operand planes
  // gradient pass over prepared weights (grad_v2.hip): tiles of 128 lines x 128 inputs in operand order
  const unsigned char* prep_gtiles;
  // The min/max grid of Eq. (1) (ASYM kernel variant): grid.qmax = 2^b - 1 levels, grid.qmin = 0; the scale
  // comes from the group's range, codes count from its minimum.  The surrogate and the arg-max records stay on
  // the group absmax.  mins: like scales (may be null).  Long groups: the record sweep also writes every
  // segment's (min, max), combined per group into grec_mm.
  int asym;                 // run the ASYM variant
  float* mins;
  float2* rec_mm;           // [nseg][nlines] (record sweep of the long-group variant)
  const float2* grec_mm;    // [groups][nlines] (loss sweep with gspan > 1)
};

__device__ __forceinline__ int64_t chunk_begin(int64_t w, int64_t n_mt, int64_t nwg) {
  return (w * n_mt) / nwg;
}

// (x0, x1) -> packed bfloat16 pair (round to nearest even), x0 in the low half
__device__ __forceinline__ uint32_t pack_bf16(float x0, float x1) {
  floatx2 v = {x0, x1};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf16_lo_f32(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi_f32(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  uintx4 v = {a, b, c, d};
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ bf16x8 as_bf16x8(uintx4 v) { return __builtin_bit_cast(bf16x8, v); }

#define CAFEQ_MFMA_BF16(A, B, C) __builtin_amdgcn_mfma_f32_32x32x16_bf16((A), (B), (C), 0, 0, 0)

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ halfx8 as_halfx8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  uintx4 v = {a, b, c, d};
  return __builtin_bit_cast(halfx8, v);
}
__device__ __forceinline__ halfx8 as_halfx8(uintx4 v) { return __builtin_bit_cast(halfx8, v); }
#define CAFEQ_MFMA_F16(A, B, C) __builtin_amdgcn_mfma_f32_32x32x16_f16((A), (B), (C), 0, 0, 0)

// s_waitcnt vmcnt(n) for a value of n that is a compile-time constant after unrolling (n is
// clamped to the counter's 6 bits; a smaller n only waits for more).
#define CAFEQ_VMW(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
__device__ __forceinline__ void vm_wait(int n) {
  switch (n > 63 ? 63 : n) {
    CAFEQ_VMW(0) CAFEQ_VMW(1) CAFEQ_VMW(2) CAFEQ_VMW(3) CAFEQ_VMW(4) CAFEQ_VMW(5) CAFEQ_VMW(6) CAFEQ_VMW(7)
    CAFEQ_VMW(8) CAFEQ_VMW(9) CAFEQ_VMW(10) CAFEQ_VMW(11) CAFEQ_VMW(12) CAFEQ_VMW(13) CAFEQ_VMW(14) CAFEQ_VMW(15)
    CAFEQ_VMW(16) CAFEQ_VMW(17) CAFEQ_VMW(18) CAFEQ_VMW(19) CAFEQ_VMW(20) CAFEQ_VMW(21) CAFEQ_VMW(22) CAFEQ_VMW(23)
    CAFEQ_VMW(24) CAFEQ_VMW(25) CAFEQ_VMW(26) CAFEQ_VMW(27) CAFEQ_VMW(28) CAFEQ_VMW(29) CAFEQ_VMW(30) CAFEQ_VMW(31)
    CAFEQ_VMW(32) CAFEQ_VMW(33) CAFEQ_VMW(34) CAFEQ_VMW(35) CAFEQ_VMW(36) CAFEQ_VMW(37) CAFEQ_VMW(38) CAFEQ_VMW(39)
    CAFEQ_VMW(40) CAFEQ_VMW(41) CAFEQ_VMW(42) CAFEQ_VMW(43) CAFEQ_VMW(44) CAFEQ_VMW(45) CAFEQ_VMW(46) CAFEQ_VMW(47)
    CAFEQ_VMW(48) CAFEQ_VMW(49) CAFEQ_VMW(50) CAFEQ_VMW(51) CAFEQ_VMW(52) CAFEQ_VMW(53) CAFEQ_VMW(54) CAFEQ_VMW(55)
    CAFEQ_VMW(56) CAFEQ_VMW(57) CAFEQ_VMW(58) CAFEQ_VMW(59) CAFEQ_VMW(60) CAFEQ_VMW(61) CAFEQ_VMW(62)
    default: asm volatile("s_waitcnt vmcnt(63)" ::: "memory"); break;
  }
}
#undef CAFEQ_VMW

// Weights of one strip (32 lines x one segment of L axis indices): element j(f, h) = 8(f/4) + 4h + f%4
// of the lane's line goes to wreg[f].  Lines beyond the matrix re-read the last line and are zeroed.
template <int L, int AXIS>
__device__ __forceinline__ void load_strip(const CoreParams& p, float (&wreg)[L / 2], int seg, int mis, int wave,
                                           int ln, int h) {
  const int64_t line = int64_t(mis) * kMacroLines + wave * kStripLines + ln;
  const bool valid = line < p.nlines;
  const int64_t lc = valid ? line : p.nlines - 1;   // out-of-range lanes re-read the last line, then zero it
  const int64_t ax0 = int64_t(seg) * L;
  if (AXIS == CAFEQ_AXIS_COL) {
    if (p.dtype == CAFEQ_F32) {
      const float* src = static_cast<const float*>(p.W) + lc * p.ld + ax0 + 4 * h;
#pragma unroll
      for (int c = 0; c < L / 8; ++c) {
        const float4 v = *reinterpret_cast<const float4*>(src + 8 * c);
        wreg[4 * c] = v.x; wreg[4 * c + 1] = v.y; wreg[4 * c + 2] = v.z; wreg[4 * c + 3] = v.w;
      }
    } else {
      const uint16_t* src = static_cast<const uint16_t*>(p.W) + lc * p.ld + ax0 + 4 * h;
#pragma unroll
      for (int c = 0; c < L / 8; ++c) {
        const float4 v = load4(src + 8 * c);
        wreg[4 * c] = v.x; wreg[4 * c + 1] = v.y; wreg[4 * c + 2] = v.z; wreg[4 * c + 3] = v.w;
      }
    }
  } else {
    // uniform row pointer (bumped by the leading dimension) + 32-bit lane offset
    const uint32_t loff = uint32_t(int64_t(4 * h) * p.ld + lc);
    if (p.dtype == CAFEQ_F32) {
      const float* rp = static_cast<const float*>(p.W) + ax0 * p.ld;
#pragma unroll
      for (int c = 0; c < L / 8; ++c) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wreg[4 * c + e] = rp[loff];
          rp += p.ld;
        }
        rp += 4 * p.ld;
      }
    } else {
      const uint16_t* rp = static_cast<const uint16_t*>(p.W) + ax0 * p.ld;
#pragma unroll
      for (int c = 0; c < L / 8; ++c) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wreg[4 * c + e] = bf16_bits_to_f32(rp[loff]);
          rp += p.ld;
        }
        rp += 4 * p.ld;
      }
    }
  }
  if (!valid) {
#pragma unroll
    for (int f = 0; f < L / 2; ++f) wreg[f] = 0.f;
  }
}

// GRAD = false compiles the gradient out: for segments of up to 128 that variant fits in half
// the register file and needs no weight staging area, so two workgroups share a compute unit
// (two waves per SIMD).
// F16 (gradient-free variant, one block per segment): the forward contraction runs on two-part
// half-precision operands -- the strip's weights scaled per line, the transform block scaled per block,
// each by a power of two that puts its largest magnitude into [2^14, 2^15) -- with three part products
// (hi.hi, hi.lo, lo.hi; relative error per term below 2^-20, the same order as the float32
// accumulation) instead of six bfloat16 ones; the accumulators are scaled back before anything reads
// them.  The inverse transform keeps the bfloat16 parts.
// LONGG: the variant for groups that span several segments (CoreParams::gspan; one group per segment inside
// the kernel): its record-only sweep and its loss sweep with the group's absmax taken from the combined records.
// ASYM: the min/max grid of Eq. (1) instead of the symmetric absmax grid (gradient-free variants only: the
// gradient of the surrogate depends on the grid through a constant alone and runs from the records).
template <int K, int G, int AXIS, bool GRAD, bool F16 = false, bool LONGG = false, bool ASYM = false>
__global__ __launch_bounds__(kThreads, (!GRAD && Geo<K, G>::L <= 128) ? 2 : 1) void xform_core_kernel(const CoreParams p) {
  static_assert(!F16 || (!GRAD && Geo<K, G>::NBLK == 1), "half-precision forward: gradient-free, one block per segment");
  static_assert(!ASYM || (!GRAD && !F16), "min/max grid: gradient-free, full-precision forward");
  static_assert(!LONGG || (!GRAD && Geo<K, G>::NGRP == 1), "long groups: gradient-free, one group per segment");
  using g = Geo<K, G>;
  constexpr bool GRAD_ON = GRAD && g::GRAD_OK;
  constexpr int GTN = GRAD_ON ? g::GT : 1;
  constexpr int L = g::L, NT = g::NT, KT = g::KT, NGRP = g::NGRP, RPG = g::RPG, NBLK = g::NBLK;
  constexpr int PLANEB = g::PLANEB, STAGEB = g::STAGEB, NSTG = g::RING_STAGES;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* ring = smem;
  unsigned char* wst = smem + g::RINGB;                                   // only if do_grad
  int16_t* jst = reinterpret_cast<int16_t*>(wst + 2 * g::WST_PLANEB);     // [NGRP][128 lines]
  uint32_t* cfp = reinterpret_cast<uint32_t*>(wst + 2 * g::WST_PLANEB + NGRP * kMacroLines * 2);
  float* hred = reinterpret_cast<float*>(smem + g::RINGB + (p.do_grad ? g::GRADB : 0));  // [kNW][kHdrFloats]
  float* wmax = hred + kNW * kHdrFloats;                                  // [kNW]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // the same value, known to be wave-uniform
  const int ln = lane & 31, h = lane >> 5;

  // contiguous chunks; consecutive chunks on the same XCD (workgroup i runs on XCD i % 8)
  int64_t w = blockIdx.x;
  if ((p.nwg & 7) == 0) w = int64_t(blockIdx.x & 7) * (p.nwg >> 3) + (blockIdx.x >> 3);
  const int64_t mt0 = chunk_begin(w, p.n_mt, p.nwg), mt1 = chunk_begin(w + 1, p.n_mt, p.nwg);
  if (mt0 >= mt1) return;

  // The operand stages are consumed in a fixed order: for each macro-tile, the NT forward stages
  // of its segment, then (loss calls) the NT inverse stages.  The fill of the stage NSTG-1 steps
  // ahead is issued at the top of every step; which stage that is follows from the (unrolled)
  // step index, so the fetch needs no cursor: only the block ids of this macro-tile's segment
  // (cb) and of the next macro-tile's (nbk).
  const int seg_first = int(mt0 / p.mt_per_seg);
  const int mis_first = int(mt0 - int64_t(seg_first) * p.mt_per_seg);   // macro-tile within segment
  const int mt_per_seg = int(p.mt_per_seg);
  constexpr int D = NSTG - 1;
  constexpr int FWDP = F16 ? 2 : kFwdPlanes;                 // operand planes of a forward stage
  constexpr int NFW = FWDP * PLANEB / 16 / kThreads;         // loads every wave issues per forward stage
  constexpr int NIW = kInvPlanes * PLANEB / 16 / kThreads;   // ... per inverse stage (K = 32: some waves one more)
  constexpr int NWL = AXIS == CAFEQ_AXIS_COL ? L / 8 : L / 2; // load instructions of one strip's weights
  const uint32_t voff = uint32_t(tid) * 16u;
  auto blk_id = [&](int sg_, int blk) {
    const int gb = sg_ * NBLK + blk;
    return (AXIS == CAFEQ_AXIS_ROW && p.rep != 1) ? gb / p.rep : gb;
  };
  // Asynchronous copy of stage s of block bid (np planes of K x 32 bf16, contiguous and already
  // swizzled) from global memory (L2) into ring stage dst_stage with the LDS-DMA load: 16 bytes
  // per lane, lane i of a wave lands at base + 16 i; no registers, no LDS store instructions.
  // Issued as opaque assembly on purpose: the compiler would otherwise drain every outstanding
  // load before each later LDS read (it cannot see that the ring stage being filled is not the
  // one being read); completion is tracked with vm_wait() below.  The LDS byte address assumes
  // that dynamic LDS starts at 0 (the kernel has no static LDS).
  auto dma = [&](const uint16_t* base, int np, int bid, int s_, int dst_stage) {
    const unsigned char* src = reinterpret_cast<const unsigned char*>(base) +
                               (int64_t(bid) * KT + s_) * (int64_t(np) * PLANEB);
    const uint32_t dst = uint32_t(dst_stage) * STAGEB + uint32_t(wave_u) * 1024u;
    const int nch = np * (PLANEB / 16);
#pragma unroll
    for (int i = 0; i < g::A_VEC_PER_THREAD; ++i) {
      if (i * kThreads + 3 * 64 < nch || i * kThreads + wave_u * 64 < nch) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(dst + uint32_t(i) * 4096u), "v"(voff), "s"(src + i * 4096) : "memory");
      }
    }
  };
  int cb[NBLK], nbk[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i) cb[i] = nbk[i] = blk_id(seg_first, i);

  dma(p.Afwd, FWDP, cb[0], 0, 0);
  if (D == 2) dma(p.Afwd, FWDP, cb[1 / KT], 1 % KT, 1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // running partial sums (per lane)
  float s_l2 = 0.f, s_errz = 0.f, s_wsq = 0.f, s_sur = 0.f;
  float s_va2[NGRP];
#pragma unroll
  for (int i = 0; i < NGRP; ++i) s_va2[i] = 0.f;
  float m_ref = -INFINITY;  // kLossLse: reference of this workgroup's exponentials

  // gradient tiles of this wave: tile rows r = wave, wave + 4, ... (< NT), KT tiles each;
  // element [j = r*32 + 8(v/4)+4h+v%4][m = mt*32 + ln] of the segment's k x k blocks
  floatx16 gt[GTN];
#pragma unroll
  for (int i = 0; i < GTN; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) gt[i][v] = 0.f;

  int cur_seg = seg_first;
  int stage = 0;       // ring stage being consumed

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
    __syncthreads();
    if (tid < kHdrVa2 + NGRP) {
      float t = 0.f;
#pragma unroll
      for (int ww = 0; ww < kNW; ++ww) t += hred[ww * kHdrFloats + tid];
      if (tid == kHdrMref) t = m_ref;
      p.slot_hdr[slot * kHdrFloats + tid] = t;
    }
    if constexpr (GRAD_ON) if (p.do_grad) {
      float* dst = p.slot_grad + slot * int64_t(NBLK * K * K);
#pragma unroll
      for (int gr = 0; gr < g::GT_ROWS; ++gr) {
        const int r = wave + gr * kNW;                 // tile row within the segment
        if (r < NT) {
          const int blk = r / KT, jt = r % KT;
#pragma unroll
          for (int mt_ = 0; mt_ < KT; ++mt_) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int j = jt * 32 + 8 * (v / 4) + 4 * h + (v % 4);
              dst[(blk * K + j) * K + mt_ * 32 + ln] = gt[gr * KT + mt_][v];
              gt[gr * KT + mt_][v] = 0.f;
            }
          }
        }
      }
    }
    __syncthreads();
    s_l2 = s_errz = s_wsq = s_sur = 0.f;
#pragma unroll
    for (int i = 0; i < NGRP; ++i) s_va2[i] = 0.f;
    m_ref = -INFINITY;
  };

  // ---- weights of a strip, loaded one macro-tile ahead (after the last use of the previous
  // strip's weights)
  float wreg[L / 2];
  auto load_w = [&](int seg, int mis) { load_strip<L, AXIS>(p, wreg, seg, mis, wave, ln, h); };
  load_w(seg_first, mis_first);

  int seg = seg_first, mis = mis_first;
  for (int64_t mt = mt0; mt < mt1; ++mt) {
    if (seg != cur_seg) {
      if (p.do_inverse || p.do_grad) flush(cur_seg);   // partial buffers exist only for loss calls
      cur_seg = seg;
    }
    const int64_t line = int64_t(mis) * kMacroLines + wave * kStripLines + ln;
    const bool valid = line < p.nlines;
    const int64_t ax0 = int64_t(seg) * L;  // first axis index of the segment
    int nseg_ = seg, nmis = mis + 1;       // the macro-tile after this one
    if (nmis == mt_per_seg) { nmis = 0; ++nseg_; }
    // what the prefetches of this macro-tile aim at: the next macro-tile, or (last one of the
    // workgroup) this one again, so that every step issues the same loads and the waits on the
    // memory counter are compile-time constants
    const bool has_next = mt + 1 < mt1;
    const int pseg = has_next ? nseg_ : seg, pmis = has_next ? nmis : mis;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) nbk[i] = blk_id(pseg, i);
    // All of this strip's weights are needed within the next few steps; waiting for the last of
    // them here (one wait) keeps the compiler from draining the in-flight ring fills later, at
    // the first use of each late register.
    asm volatile("" :: "v"(wreg[L / 2 - 1]));

    // ---- forward transform.  One ring stage = 32 inputs (two MFMA steps) of one block; every
    // step the lane splits its eight weights exactly into bfloat16 parts (hi + mid + lo), feeds
    // them to all KT output tiles of the block, and (gradient calls) parks the hi/mid parts in
    // the LDS staging area transposed, [input m][line], for the gradient contraction over lines.
    // F16: power-of-two scale of this line's weights (largest magnitude of the segment -> [2^14, 2^15))
    // and the factor that takes the accumulators back (times the block's own factor)
    float wsc = 1.f, usc = 1.f;
    if constexpr (F16) {
      float m = 0.f;
#pragma unroll
      for (int f = 0; f < L / 2; ++f) m = fmaxf(m, fabsf(wreg[f]));
      m = fmaxf(m, __shfl_xor(m, 32));
      int e = int(__float_as_uint(m) >> 23);     // biased exponent
      e = e < 32 ? 32 : (e > 254 ? 254 : e);     // lines of (almost) zeros: any scale will do
      wsc = __uint_as_float(uint32_t(268 - e) << 23);          // 2^(14 - (e - 127))
      usc = __uint_as_float(uint32_t(e - 14) << 23) * p.fscale[cb[0]];
    }
    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    const int swz = (ln >> 2) & 3;
    const int aoff0 = ln * 64 + ((h ^ swz) << 4), aoff1 = ln * 64 + (((2 + h) ^ swz) << 4);
    unsigned char* wcol = wst + (wave * kStripLines + ln) * 2;
#pragma unroll
    for (int sg = 0; sg < NT; ++sg) {               // stage = 32 inputs; sg / KT is the block
      int nw = NFW;
      {
        const int tq = sg + D, dst = stage == 0 ? NSTG - 1 : stage - 1;
        if (tq < NT) {
          dma(p.Afwd, FWDP, cb[tq / KT], tq % KT, dst);
        } else {
          nw = NIW;
          if (p.do_inverse) dma(p.Ainv, kInvPlanes, cb[(tq - NT) / KT], (tq - NT) % KT, dst);
          else dma(p.Afwd, FWDP, nbk[(tq - NT) / KT], (tq - NT) % KT, dst);
        }
      }
      const unsigned char* sbase = ring + stage * STAGEB;
      const int blk = sg / KT;
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2) {
        const int c = 2 * sg + c2;                   // MFMA step within the segment: inputs 16c..16c+15
        if constexpr (F16) {
          uint32_t bh[4], bl[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float x0 = wreg[8 * c + 2 * i], x1 = wreg[8 * c + 2 * i + 1];
            if (p.do_inverse) s_wsq = fmaf(x0, x0, fmaf(x1, x1, s_wsq));
            const float y0 = x0 * wsc, y1 = x1 * wsc;
            const auto hh = __builtin_amdgcn_cvt_pkrtz(y0, y1);
            const auto hl = __builtin_amdgcn_cvt_pkrtz(y0 - float(hh[0]), y1 - float(hh[1]));
            bh[i] = __builtin_bit_cast(uint32_t, hh);
            bl[i] = __builtin_bit_cast(uint32_t, hl);
          }
          const halfx8 vbh = as_halfx8(bh[0], bh[1], bh[2], bh[3]);
          const halfx8 vbl = as_halfx8(bl[0], bl[1], bl[2], bl[3]);
          const int ao = c2 == 0 ? aoff0 : aoff1;
          halfx8 xh[KT], xl[KT];
#pragma unroll
          for (int t = 0; t < KT; ++t) {
            const unsigned char* ap = sbase + t * (32 * 64) + ao;
            xh[t] = as_halfx8(*reinterpret_cast<const uintx4*>(ap));
            xl[t] = as_halfx8(*reinterpret_cast<const uintx4*>(ap + PLANEB));
          }
#pragma unroll
          for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_F16(xl[t], vbh, acc[blk * KT + t]);
#pragma unroll
          for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_F16(xh[t], vbl, acc[blk * KT + t]);
#pragma unroll
          for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_F16(xh[t], vbh, acc[blk * KT + t]);
        } else {
        uint32_t bh[4], bm[4], bl[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float x0 = wreg[8 * c + 2 * i], x1 = wreg[8 * c + 2 * i + 1];
          if (p.do_inverse) s_wsq = fmaf(x0, x0, fmaf(x1, x1, s_wsq));
          const uint32_t ph = pack_bf16(x0, x1);
          const float r0 = x0 - bf16_lo_f32(ph), r1 = x1 - bf16_hi_f32(ph);
          const uint32_t pm = pack_bf16(r0, r1);
          bh[i] = ph; bm[i] = pm;
          bl[i] = pack_bf16(r0 - bf16_lo_f32(pm), r1 - bf16_hi_f32(pm));
        }
        if constexpr (GRAD_ON) if (p.do_grad) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int m0 = 16 * c + 8 * (i / 2) + 4 * h + 2 * (i % 2);   // inputs of the packed pair: m0, m0+1
            unsigned char* r0 = wcol + m0 * g::WST_ROWB;
            *reinterpret_cast<uint16_t*>(r0) = uint16_t(bh[i]);
            *reinterpret_cast<uint16_t*>(r0 + g::WST_ROWB) = uint16_t(bh[i] >> 16);
            *reinterpret_cast<uint16_t*>(r0 + g::WST_PLANEB) = uint16_t(bm[i]);
            *reinterpret_cast<uint16_t*>(r0 + g::WST_PLANEB + g::WST_ROWB) = uint16_t(bm[i] >> 16);
          }
        }
        const bf16x8 vbh = as_bf16x8(bh[0], bh[1], bh[2], bh[3]);
        const bf16x8 vbm = as_bf16x8(bm[0], bm[1], bm[2], bm[3]);
        const bf16x8 vbl = as_bf16x8(bl[0], bl[1], bl[2], bl[3]);
        const int ao = c2 == 0 ? aoff0 : aoff1;
        bf16x8 xh[KT], xm[KT], xl[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t) {
          const unsigned char* ap = sbase + t * (32 * 64) + ao;
          xh[t] = as_bf16x8(*reinterpret_cast<const uintx4*>(ap));
          xm[t] = as_bf16x8(*reinterpret_cast<const uintx4*>(ap + PLANEB));
          xl[t] = as_bf16x8(*reinterpret_cast<const uintx4*>(ap + 2 * PLANEB));
        }
        // six products, smallest terms first; the KT tiles interleaved so that consecutive MFMAs
        // are independent
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_BF16(xl[t], vbh, acc[blk * KT + t]);
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_BF16(xh[t], vbl, acc[blk * KT + t]);
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_BF16(xm[t], vbm, acc[blk * KT + t]);
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_BF16(xm[t], vbh, acc[blk * KT + t]);
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_BF16(xh[t], vbm, acc[blk * KT + t]);
#pragma unroll
        for (int t = 0; t < KT; ++t) acc[blk * KT + t] = CAFEQ_MFMA_BF16(xh[t], vbh, acc[blk * KT + t]);
        }
      }
      // The stage consumed D steps from now was issued D - 1 steps ago and must have landed
      // before the barrier.  Loads complete in order, so it has once only younger loads are
      // pending: this step's fill when D = 2, nothing when D = 1.
      vm_wait(D == 2 ? nw : 0);
      __syncthreads();
      stage = stage == NSTG - 1 ? 0 : stage + 1;
    }
    if constexpr (F16) {
      // back to the units of Z: exact (powers of two) unless the result leaves the float32 range
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] *= usc;
    }

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
        // uniform row pointer (bumped by whole rows) + 32-bit lane offset
        const uint32_t loff = uint32_t(4 * h) * uint32_t(p.cols) + uint32_t(line);
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float* rowp = p.Zout + (ax0 + 32 * t + 8 * (v / 4) + (v % 4)) * p.cols;
            rowp[loff] = acc[t][v];
          }
      }
    }

    float err[L / 2];   // quantization error E = dequant(Q(Z)) - Z, same layout as the accumulators
    const bool want_q = p.codes || p.scales || p.do_inverse || (LONGG && p.rec);
    const bool big = LONGG && p.gspan > 1;                           // the group spans several segments
    const bool first_of_group = !big || seg % p.gspan == 0;          // group-level sums are taken once
    const bool lse_on = p.loss_kind == kLossLse && p.do_inverse;
    if (want_q) {
      // ---- per-group absmax (+ argmax), codes, error in place
      float gz[NGRP];   // signed value at the arg-max element
      int gj[NGRP];     // its axis index inside the segment
      uint32_t qpk[L / 8];   // codes, four per register (axis indices 8*f4 + 4h .. +3)
#pragma unroll
      for (int gi = 0; gi < NGRP; ++gi) {
        float a = -1.f, zs = 0.f;
        int jf = 0;   // arg-max index without the lane-half term 4h: an immediate per register
#pragma unroll
        for (int f = gi * RPG; f < (gi + 1) * RPG; ++f) {
          const float z = acc[f / 16][f % 16];
          const float v = fabsf(z);
          if (v > a) { a = v; zs = z; jf = 8 * (f / 4) + (f % 4); }
        }
        int j = jf + 4 * h;
        const float oz = __shfl_xor(zs, 32);
        const int oj = __shfl_xor(j, 32);
        const float oa = fabsf(oz);
        if (oa > a || (oa == a && oj < j)) { a = oa; zs = oz; j = oj; }
        float mn = 0.f, mx = 0.f;   // ASYM: the group's minimum and maximum
        if constexpr (ASYM) {
          mn = mx = acc[(gi * RPG) / 16][(gi * RPG) % 16];
#pragma unroll
          for (int f = gi * RPG + 1; f < (gi + 1) * RPG; ++f) {
            mn = fminf(mn, acc[f / 16][f % 16]);
            mx = fmaxf(mx, acc[f / 16][f % 16]);
          }
          mn = fminf(mn, __shfl_xor(mn, 32));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
        }
        if (p.rec && valid && h == 0) {   // index relative to the group's first element
          p.rec[(int64_t(seg) * NGRP + gi) * p.nlines + line] = make_float2(zs, __int_as_float(j - gi * G));
          if constexpr (ASYM && LONGG) if (p.rec_mm) p.rec_mm[int64_t(seg) * p.nlines + line] = make_float2(mn, mx);
        }
        if constexpr (LONGG) if (big) {
          // the group's absmax comes from the combined records (NGRP == 1 here)
          const int64_t at = int64_t(seg / p.gspan) * p.nlines + (valid ? line : p.nlines - 1);
          const float2 r = p.grec[at];
          zs = valid ? r.x : 0.f;
          a = fabsf(zs);
          if constexpr (ASYM) {
            const float2 mm = p.grec_mm[at];
            mn = valid ? mm.x : 0.f;
            mx = valid ? mm.y : 0.f;
          }
        }
        gz[gi] = zs; gj[gi] = j;
        if constexpr (LONGG) if (!(p.codes || p.scales || p.do_inverse)) continue;   // record-only sweep
        // symmetric grid: steps of absmax / qmax around zero; Eq. (1): steps of (max - min) / levels from min
        const float span = ASYM ? mx - mn : a;
        const float inv = grid_inv(span, p.grid.qmax);
        const float s = grid_scale(span, p.grid.qmax);
        if (p.scales && valid && h == 0 && first_of_group) {
          int64_t at;
          if (big) {
            const int64_t gidx = seg / p.gspan, ng = p.nseg / p.gspan;
            at = AXIS == CAFEQ_AXIS_COL ? line * ng + gidx : gidx * p.cols + line;
          } else {
            const int64_t gidx = ax0 / G + gi;   // group index along the axis
            at = AXIS == CAFEQ_AXIS_COL ? line * (p.cols / G) + gidx : gidx * p.cols + line;
          }
          p.scales[at] = s;
          if constexpr (ASYM) if (p.mins) p.mins[at] = mn;
        }
#pragma unroll
        for (int f4 = gi * RPG / 4; f4 < (gi + 1) * RPG / 4; ++f4) {
          float q[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int f = 4 * f4 + e;
            const float z = acc[f / 16][f % 16];
            float er;
            if constexpr (ASYM) {
              q[e] = grid_code(z - mn, inv, p.grid);
              er = __fadd_rn(__fmul_rn(q[e], s), mn) - z;
            } else {
              q[e] = grid_code(z, inv, p.grid);
              er = __fmul_rn(q[e], s) - z;
            }
            s_errz = fmaf(er, er, s_errz);
            err[f] = er;
          }
          qpk[f4] = pack4(q[0], q[1], q[2], q[3]);
        }
        if (p.do_inverse) {
          const float a2 = a * a;
          if (h == 0) s_va2[gi] += a2;
          if (p.loss_kind == kLossSur && h == 0) s_sur = fmaf(a2, p.rG[seg * NGRP + gi], s_sur);
        }
      }

      if (p.codes && valid) {
#pragma unroll
        for (int f4 = 0; f4 < L / 8; ++f4) {
          const int j0 = 8 * f4 + 4 * h;
          if (AXIS == CAFEQ_AXIS_COL) {
            *reinterpret_cast<uint32_t*>(p.codes + line * p.cols + ax0 + j0) = qpk[f4];
          } else {
            // uniform row pointer + 32-bit lane offset
            int8_t* rowp = p.codes + (ax0 + 8 * f4) * p.cols;
            const uint32_t loff = uint32_t(4 * h) * uint32_t(p.cols) + uint32_t(line);
#pragma unroll
            for (int e = 0; e < 4; ++e) rowp[loff + uint32_t(e) * uint32_t(p.cols)] = int8_t(qpk[f4] >> (8 * e));
          }
        }
      }

      // ---- LogSumExp bookkeeping: exponentials relative to a workgroup-wide running reference
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
          if constexpr (GRAD_ON) if (p.do_grad) {
#pragma unroll
            for (int i = 0; i < GTN; ++i)
#pragma unroll
              for (int v = 0; v < 16; ++v) gt[i][v] *= sc;
          }
          s_sur *= sc;
          m_ref = nm;
        }
        __syncthreads();
      }

      // ---- gradient through Z: stage this strip's W parts and (arg-max, coefficient) pairs
      if (p.do_grad || lse_on) {
#pragma unroll
        for (int gi = 0; gi < NGRP; ++gi) {
          float coef;
          if (p.loss_kind == kLossSur) {
            coef = 2.f * p.beta * p.rG[seg * NGRP + gi] * gz[gi];
          } else {
            const float e = valid ? __expf(p.lse_t * (fabsf(gz[gi]) - m_ref)) : 0.f;
            if (h == 0 && first_of_group) s_sur += e;
            coef = gz[gi] < 0.f ? -e : e;
          }
          if (GRAD_ON && p.do_grad && h == 0) {
            // coefficient as an exact-to-16-bit bfloat16 pair (hi in the low half, lo in the high half)
            const uint32_t ch = pack_bf16(coef, 0.f);
            const uint32_t cl = pack_bf16(coef - bf16_lo_f32(ch), 0.f);
            jst[gi * kMacroLines + wave * kStripLines + ln] = int16_t(gj[gi]);
            cfp[gi * kMacroLines + wave * kStripLines + ln] = (ch & 0xFFFFu) | (cl << 16);
          }
        }
      }
      if constexpr (GRAD_ON) if (p.do_grad) {
        // (the W hi/mid parts were staged during the forward phase)
        __syncthreads();
        // G[j][m] += sum over the 128 lines of S[line][j] * W[line][m], 16 lines per MFMA step
#pragma unroll
        for (int gr = 0; gr < g::GT_ROWS; ++gr) {
          const int r = wave + gr * kNW;
          if (r < NT) {
            const int jrow = r * 32 + ln;              // this lane's row of S^T
            const int gi = jrow / G;                   // its group (uniform over the tile: G >= 32)
            const int blk = r / KT;
#pragma unroll
            for (int s = 0; s < kMacroLines / 16; ++s) {
              const int l0 = 16 * s + 8 * h;
              // eight lines' arg-max indices and packed coefficients
              const uintx4 jv = *reinterpret_cast<const uintx4*>(jst + gi * kMacroLines + l0);
              const uintx4 c0 = *reinterpret_cast<const uintx4*>(cfp + gi * kMacroLines + l0);
              const uintx4 c1 = *reinterpret_cast<const uintx4*>(cfp + gi * kMacroLines + l0 + 4);
              uint32_t sel[8];
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const int js = int((jv[e / 2] >> (16 * (e % 2))) & 0xFFFFu);
                const uint32_t cv = e < 4 ? c0[e] : c1[e - 4];
                sel[e] = js == jrow ? cv : 0u;
              }
              uintx4 sh, sl;
#pragma unroll
              for (int e2 = 0; e2 < 4; ++e2) {
                sh[e2] = __builtin_amdgcn_perm(sel[2 * e2 + 1], sel[2 * e2], 0x05040100u);
                sl[e2] = __builtin_amdgcn_perm(sel[2 * e2 + 1], sel[2 * e2], 0x07060302u);
              }
              const bf16x8 ash = as_bf16x8(sh), asl = as_bf16x8(sl);
              // operands of all KT tiles first, then the three part products tile-interleaved, so that
              // consecutive MFMAs never wait on each other's accumulator
              bf16x8 bh[KT], bm[KT];
#pragma unroll
              for (int mt_ = 0; mt_ < KT; ++mt_) {
                const unsigned char* wrow = wst + (blk * K + mt_ * 32 + ln) * g::WST_ROWB + l0 * 2;
                bh[mt_] = as_bf16x8(*reinterpret_cast<const uintx4*>(wrow));
                bm[mt_] = as_bf16x8(*reinterpret_cast<const uintx4*>(wrow + g::WST_PLANEB));
              }
#pragma unroll
              for (int mt_ = 0; mt_ < KT; ++mt_) gt[gr * KT + mt_] = CAFEQ_MFMA_BF16(asl, bh[mt_], gt[gr * KT + mt_]);
#pragma unroll
              for (int mt_ = 0; mt_ < KT; ++mt_) gt[gr * KT + mt_] = CAFEQ_MFMA_BF16(ash, bm[mt_], gt[gr * KT + mt_]);
#pragma unroll
              for (int mt_ = 0; mt_ < KT; ++mt_) gt[gr * KT + mt_] = CAFEQ_MFMA_BF16(ash, bh[mt_], gt[gr * KT + mt_]);
            }
          }
        }
      }
    }

    // ---- the next strip's weights: wreg and the W parts are dead from here on (the staged
    // copy is read by the other waves, protected by the barriers of the inverse phase)
    if (!p.do_inverse) load_w(pseg, pmis);

    // ---- inverse transform of the error and the l2 proxy: same stage order; the error registers
    // 8c..8c+7 of the lane are the B operand of step c, split on the fly into hi + mid
    if (p.do_inverse) {
      // B operand of MFMA step c: the lane's error registers 8c..8c+7 as bfloat16 hi and mid parts
      auto split_e = [&](int c, bf16x8& vh, bf16x8& vm) {
        uint32_t eh[4], em[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int f0 = 8 * c + 2 * i;
          const float x0 = err[f0], x1 = err[f0 + 1];
          const uint32_t ph = pack_bf16(x0, x1);
          eh[i] = ph;
          em[i] = pack_bf16(x0 - bf16_lo_f32(ph), x1 - bf16_hi_f32(ph));
        }
        vh = as_bf16x8(eh[0], eh[1], eh[2], eh[3]);
        vm = as_bf16x8(em[0], em[1], em[2], em[3]);
      };
#pragma unroll
      for (int blk = 0; blk < NBLK; ++blk) {
        floatx16 d[KT];
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) d[t][v] = 0.f;
        bf16x8 veh, vem;
        split_e(2 * blk * KT, veh, vem);
#pragma unroll
        for (int s2 = 0; s2 < KT; ++s2) {
          const int sg = blk * KT + s2;
          int nw = NIW;
          {
            const int tq = sg + D, dst = stage == 0 ? NSTG - 1 : stage - 1;
            if (tq < NT) {
              dma(p.Ainv, kInvPlanes, cb[tq / KT], tq % KT, dst);
            } else {
              nw = NFW;
              dma(p.Afwd, FWDP, nbk[(tq - NT) / KT], (tq - NT) % KT, dst);
            }
          }
          // The next strip's weights, right behind the first inverse stage's fill: they are
          // younger than that fill, so the two following waits may leave them pending.
          if (sg == 0) load_w(pseg, pmis);
          const unsigned char* sbase = ring + stage * STAGEB;
#pragma unroll
          for (int c2 = 0; c2 < 2; ++c2) {
            const int c = 2 * sg + c2;
            const int ao = c2 == 0 ? aoff0 : aoff1;
            bf16x8 xh[KT], xm[KT];
#pragma unroll
            for (int t = 0; t < KT; ++t) {
              const unsigned char* ap = sbase + t * (32 * 64) + ao;
              xh[t] = as_bf16x8(*reinterpret_cast<const uintx4*>(ap));
              xm[t] = as_bf16x8(*reinterpret_cast<const uintx4*>(ap + PLANEB));
            }
            __builtin_amdgcn_sched_barrier(0);   // all operand reads in flight before the first MFMA
            // the next step's operand split runs in the shadow of this step's MFMAs
            bf16x8 nveh = veh, nvem = vem;
            const bool more = !(s2 == KT - 1 && c2 == 1);
            if (more) split_e(c + 1, nveh, nvem);
#pragma unroll
            for (int t = 0; t < KT; ++t) d[t] = CAFEQ_MFMA_BF16(xm[t], veh, d[t]);
#pragma unroll
            for (int t = 0; t < KT; ++t) d[t] = CAFEQ_MFMA_BF16(xh[t], vem, d[t]);
#pragma unroll
            for (int t = 0; t < KT; ++t) d[t] = CAFEQ_MFMA_BF16(xh[t], veh, d[t]);
            // requested issue order: one MFMA, then three vector instructions of the split
#pragma unroll
            for (int i = 0; i < 3 * KT; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
            }
            veh = nveh; vem = nvem;
          }
          vm_wait((D == 2 ? nw : 0) + (sg < D ? NWL : 0));   // the weights loads are younger for D steps
          __syncthreads();
          stage = stage == NSTG - 1 ? 0 : stage + 1;
        }
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) s_l2 = fmaf(d[t][v], d[t][v], s_l2);
      }
    }
    seg = nseg_;
    mis = nmis;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) cb[i] = nbk[i];
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the last macro-tile's (unused) prefetches
  if (p.do_inverse || p.do_grad) flush(cur_seg);
}

}  // namespace cafeq
