// Gradient pass of the two-pass scheme: gradT_b += W_b^T S_b (columns) / S_b W_b^T (rows), where
// S has one non-zero per (line, group), at the group's arg-max, recorded by the gradient-free
// pass of the fused kernel.  (Paper Sec. 4.1: gradient of the surrogate through the transformed
// weights; Sec. 4.2: of the LogSumExp surrogate.)
//
// The axis is cut into chunks of 128 inputs.  A workgroup owns a contiguous, chunk-major range of
// macro-tiles (128 lines x one chunk), a wave 32 lines.  Per macro-tile the waves split their
// weights exactly into bfloat16 hi + mid parts and park them in LDS transposed, [input m][line];
// then every wave accumulates its tile rows (32 outputs j each) of the k x k gradient blocks the
// chunk's inputs belong to, over the 128 lines, on the matrix cores (three part products, float32
// accumulation, operands: S^T built in registers from the records, W parts from LDS):
//   K <= 128: the chunk holds 128 / K whole blocks; tile row r (r = wave) lies in block 32 r / K and has
//             K / 32 tiles (the block's inputs);
//   K == 256: the chunk is one half of a block's inputs; all eight tile rows of the block (two per
//             wave) meet it, four tiles each -- the two halves are different chunks, so every weight
//             is still read once.
// The group length is a run-time value (any multiple of 32, whole channels included): a tile row of
// 32 outputs lies inside one group, whose record (signed value at the arg-max, index inside the
// group) decides whether and where the line's coefficient falls into the row.
// One partial per (workgroup, chunk) -- [128 or 256 outputs][K or 128 inputs] -- reduced in fixed
// order by reduce_grad_kernel.
#pragma once
#include "xform_core.hpp"

namespace cafeq {

// The weights of one strip, fetched in L/8 chunks of four axis indices each (same register
// layout as load_strip) so that the loads can be spread over the matrix-core phase of the
// previous macro-tile.  begin() fixes the strip, chunk(c) must be called for c = 0 .. L/8-1 in
// order, finish() zeroes the lines beyond the matrix.
template <int L, int AXIS>
struct StripLoader {
  const CoreParams& p;
  float (&wreg)[L / 2];
  const unsigned char* rp;   // AXIS_ROW: uniform row pointer, bumped as the chunks go by
  const unsigned char* lp;   // AXIS_COL: this lane's line
  uint32_t loff;
  bool valid;
  __device__ __forceinline__ StripLoader(const CoreParams& p_, float (&w_)[L / 2]) : p(p_), wreg(w_) {}
  __device__ __forceinline__ void begin(int seg, int mis, int wave, int ln, int h) {
    const int64_t line = int64_t(mis) * kMacroLines + wave * kStripLines + ln;
    valid = line < p.nlines;
    const int64_t lc = valid ? line : p.nlines - 1;
    const int64_t ax0 = int64_t(seg) * L;
    const int es = p.dtype == CAFEQ_F32 ? 4 : 2;
    if (AXIS == CAFEQ_AXIS_COL) {
      lp = static_cast<const unsigned char*>(p.W) + (lc * p.ld + ax0 + 4 * h) * es;
    } else {
      loff = uint32_t((int64_t(4 * h) * p.ld + lc) * es);
      rp = static_cast<const unsigned char*>(p.W) + ax0 * p.ld * es;
    }
  }
  __device__ __forceinline__ void chunk(int c) {
    if (AXIS == CAFEQ_AXIS_COL) {
      float4 v;
      if (p.dtype == CAFEQ_F32) v = *reinterpret_cast<const float4*>(lp + 32 * c);
      else v = load4(reinterpret_cast<const uint16_t*>(lp + 16 * c));
      wreg[4 * c] = v.x; wreg[4 * c + 1] = v.y; wreg[4 * c + 2] = v.z; wreg[4 * c + 3] = v.w;
    } else {
      const int64_t rowb = p.ld * (p.dtype == CAFEQ_F32 ? 4 : 2);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        wreg[4 * c + e] = p.dtype == CAFEQ_F32 ? *reinterpret_cast<const float*>(rp + loff)
                                               : bf16_bits_to_f32(*reinterpret_cast<const uint16_t*>(rp + loff));
        rp += rowb;
      }
      rp += 4 * rowb;
    }
  }
  __device__ __forceinline__ void finish() {
    if (!valid) {
#pragma unroll
      for (int f = 0; f < L / 2; ++f) wreg[f] = 0.f;
    }
  }
};

template <int K>
struct GradGeo {
  static constexpr int CH = 128;                        // inputs per chunk
  static constexpr int KM = K < 128 ? K : 128;          // inputs of one tile row's block inside the chunk
  static constexpr int MT = KM / 32;                    // tiles per tile row
  static constexpr int JR = K == 256 ? 8 : 4;           // tile rows that meet a chunk
  static constexpr int JRW = JR / kNW;                  // ... per wave
  static constexpr int GT = JRW * MT;                   // accumulator tiles per wave
  static constexpr int PART = JR * 32 * KM;             // floats of one partial
  static constexpr int WST_ROWB = 2 * kMacroLines + 16;
  static constexpr int WST_PLANEB = CH * WST_ROWB;
  static constexpr int LDSB = 2 * WST_PLANEB + JR * kMacroLines * (2 + 4) + 64;
};

// (Blocks of 256: eight accumulator tiles per wave next to the 64 weight registers do not fit in half the
// register file, so that variant runs one workgroup per compute unit.)
template <int K, int AXIS>
__global__ __launch_bounds__(kThreads, K == 256 ? 1 : 2) void grad_z_kernel(const CoreParams p) {
  using g = GradGeo<K>;
  constexpr int L = g::CH, KM = g::KM, MT = g::MT, JR = g::JR, JRW = g::JRW;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* wst = smem;                                              // [2 parts][128 inputs][WST_ROWB]
  int16_t* jst = reinterpret_cast<int16_t*>(wst + 2 * g::WST_PLANEB);     // [JR][128 lines]
  uint32_t* cfp = reinterpret_cast<uint32_t*>(wst + 2 * g::WST_PLANEB + JR * kMacroLines * 2);
  float* red = reinterpret_cast<float*>(wst + 2 * g::WST_PLANEB + JR * kMacroLines * 6);   // [kNW]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5;

  int64_t w = blockIdx.x;
  if ((p.nwg & 7) == 0) w = int64_t(blockIdx.x & 7) * (p.nwg >> 3) + (blockIdx.x >> 3);
  const int64_t mt0 = chunk_begin(w, p.n_mt, p.nwg), mt1 = chunk_begin(w + 1, p.n_mt, p.nwg);

  // kLossLse: exponentials relative to the member's largest group maximum
  float m_mem = 0.f;
  if (p.loss_kind == kLossLse) {
    float m = -INFINITY;
    for (int i = tid; i < p.nslot_ref; i += kThreads) m = fmaxf(m, p.hdr_ref[int64_t(i) * kHdrFloats + kHdrMref]);
    m = cluster_allmax<64>(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m_mem = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    if (blockIdx.x == 0 && tid == 0) *p.member_ref = m_mem;
  }
  if (mt0 >= mt1) return;

  const int mt_per_seg = int(p.mt_per_seg);
  int seg = int(mt0 / p.mt_per_seg);                  // chunk of 128 inputs
  int mis = int(mt0 - int64_t(seg) * p.mt_per_seg);
  int cur_seg = seg;

  // gradient tiles of this wave: tile rows r = wave (+ 4), MT tiles each; element
  // [j = r*32 + 8(v/4)+4h+v%4][m = mt*32 + ln] of the partial
  floatx16 gt[g::GT];
#pragma unroll
  for (int i = 0; i < g::GT; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) gt[i][v] = 0.f;

  auto flush = [&](int sg_) {
    float* dst = p.slot_grad + (w + sg_) * int64_t(g::PART);
#pragma unroll
    for (int gr = 0; gr < JRW; ++gr) {
      const int r = wave + gr * kNW;
#pragma unroll
      for (int mt_ = 0; mt_ < MT; ++mt_) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int j = r * 32 + 8 * (v / 4) + 4 * h + (v % 4);
          dst[j * KM + mt_ * 32 + ln] = gt[gr * MT + mt_][v];
          gt[gr * MT + mt_][v] = 0.f;
        }
      }
    }
  };

  float wreg[L / 2];
  StripLoader<L, AXIS> loader(p, wreg);
  loader.begin(seg, mis, wave, ln, h);
#pragma unroll
  for (int c = 0; c < L / 8; ++c) loader.chunk(c);
  loader.finish();
  // The records of a strip (lanes of the first half only) are fetched with its weights: one per tile
  // row, that of the group the row's 32 outputs lie in.  joff: the row's first output inside its group.
  float2 recv[JR];
  int joff[JR];
  auto load_rec = [&](int sg_, int ms_) {
    const int64_t line = int64_t(ms_) * kMacroLines + wave * kStripLines + ln;
    const int64_t a0 = K == 256 ? int64_t(sg_ >> 1) * 256 : int64_t(sg_) * 128;   // first output of tile row 0
#pragma unroll
    for (int r = 0; r < JR; ++r) {
      const int64_t aj = a0 + 32 * r;
      const int64_t gi = aj / p.grp;
      joff[r] = int(aj - gi * p.grp);
      recv[r] = make_float2(0.f, 0.f);
      if (h == 0 && line < p.nlines) recv[r] = p.rec[gi * p.nlines + line];
    }
  };
  load_rec(seg, mis);
  // even lane: (own low half, neighbour's low half) -> row m0, lines (ln, ln+1);
  // odd lane: (neighbour's high half, own high half) -> row m0+1, lines (ln-1, ln)
  const uint32_t pair_sel = (ln & 1) ? 0x03020706u : 0x05040100u;
  unsigned char* wpair = wst + (ln & 1) * g::WST_ROWB + (wave * kStripLines + (ln & ~1)) * 2;

  for (int64_t mt = mt0; mt < mt1; ++mt) {
    if (seg != cur_seg) {
      flush(cur_seg);
      cur_seg = seg;
    }
    const int64_t line = int64_t(mis) * kMacroLines + wave * kStripLines + ln;
    const bool valid = line < p.nlines;
    int nseg_ = seg, nmis = mis + 1;
    if (nmis == mt_per_seg) { nmis = 0; ++nseg_; }

    // ---- this strip's weights as bfloat16 hi + mid parts, transposed into the staging area.
    // A lane holds (m0, m0+1) of its line; it swaps one half with the neighbouring line's lane
    // (DPP), so that the even lane owns (line, line+1) of input m0 and the odd lane of m0+1:
    // one aligned 32-bit LDS store per packed pair instead of two 16-bit ones.
#pragma unroll
    for (int c = 0; c < L / 16; ++c) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x0 = wreg[8 * c + 2 * i], x1 = wreg[8 * c + 2 * i + 1];
        const uint32_t ph = pack_bf16(x0, x1);
        const uint32_t pm = pack_bf16(x0 - bf16_lo_f32(ph), x1 - bf16_hi_f32(ph));
        const uint32_t oh = uint32_t(__builtin_amdgcn_update_dpp(0, int(ph), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
        const uint32_t om = uint32_t(__builtin_amdgcn_update_dpp(0, int(pm), 0xB1, 0xF, 0xF, true));
        const int m0 = 16 * c + 8 * (i / 2) + 4 * h + 2 * (i % 2);   // inputs of the packed pair: m0, m0+1
        unsigned char* r0 = wpair + m0 * g::WST_ROWB;
        *reinterpret_cast<uint32_t*>(r0) = __builtin_amdgcn_perm(oh, ph, pair_sel);
        *reinterpret_cast<uint32_t*>(r0 + g::WST_PLANEB) = __builtin_amdgcn_perm(om, pm, pair_sel);
      }
    }
    // ---- per tile row: where this line's arg-max falls inside the row (-1: not in it) and its coefficient
    if (h == 0) {
#pragma unroll
      for (int r = 0; r < JR; ++r) {
        float coef = 0.f;
        int jl = -1;
        if (valid) {
          const float2 rc = recv[r];
          const int jj = __float_as_int(rc.y) - joff[r];
          if (jj >= 0 && jj < 32) {
            jl = jj;
            if (p.loss_kind == kLossSur) {
              const int64_t a0 = K == 256 ? int64_t(seg >> 1) * 256 : int64_t(seg) * 128;
              coef = 2.f * p.beta * p.rG[(a0 + 32 * r) / p.grp] * rc.x;
            } else {
              const float e = __expf(p.lse_t * (fabsf(rc.x) - m_mem));
              coef = rc.x < 0.f ? -e : e;
            }
          }
        }
        // coefficient as an exact-to-16-bit bfloat16 pair (hi in the low half, lo in the high half)
        const uint32_t ch = pack_bf16(coef, 0.f);
        const uint32_t cl = pack_bf16(coef - bf16_lo_f32(ch), 0.f);
        jst[r * kMacroLines + wave * kStripLines + ln] = int16_t(jl);
        cfp[r * kMacroLines + wave * kStripLines + ln] = (ch & 0xFFFFu) | (cl << 16);
      }
    }
    // ---- the next strip's weights and records: addresses now, the loads spread over the
    // matrix-core phase below
    const bool has_next = mt + 1 < mt1;
    if (has_next) {
      loader.begin(nseg_, nmis, wave, ln, h);
      load_rec(nseg_, nmis);
    }
    __syncthreads();

    // ---- G[j][m] += sum over the 128 lines of S[line][j] * W[line][m], 16 lines per MFMA step
#pragma unroll
    for (int gr = 0; gr < JRW; ++gr) {
      const int r = wave + gr * kNW;
      const int mbase = K < 128 ? ((32 * r) / K) * K : 0;   // first input of the row's block inside the chunk
#pragma unroll
      for (int s = 0; s < kMacroLines / 16; ++s) {
        const int l0 = 16 * s + 8 * h;
        // this step's share of the next strip's weight loads (spread over the first tile row's steps)
        if (gr == 0 && has_next) {
          constexpr int per = (L / 8 + kMacroLines / 16 - 1) / (kMacroLines / 16);
#pragma unroll
          for (int c = s * per; c < (s + 1) * per && c < L / 8; ++c) loader.chunk(c);
        }
        // eight lines' positions inside this tile row and packed coefficients
        const uintx4 jv = *reinterpret_cast<const uintx4*>(jst + r * kMacroLines + l0);
        const uintx4 c0 = *reinterpret_cast<const uintx4*>(cfp + r * kMacroLines + l0);
        const uintx4 c1 = *reinterpret_cast<const uintx4*>(cfp + r * kMacroLines + l0 + 4);
        uint32_t sel[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int js = int((jv[e / 2] >> (16 * (e % 2))) & 0xFFFFu);
          const uint32_t cv = e < 4 ? c0[e] : c1[e - 4];
          sel[e] = js == ln ? cv : 0u;
        }
        uintx4 sh, sl;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          sh[e2] = __builtin_amdgcn_perm(sel[2 * e2 + 1], sel[2 * e2], 0x05040100u);
          sl[e2] = __builtin_amdgcn_perm(sel[2 * e2 + 1], sel[2 * e2], 0x07060302u);
        }
        const bf16x8 ash = as_bf16x8(sh), asl = as_bf16x8(sl);
        // operands of all MT tiles first, then the three part products tile-interleaved, so that
        // consecutive MFMAs never wait on each other's accumulator
        bf16x8 bh[MT], bm[MT];
#pragma unroll
        for (int mt_ = 0; mt_ < MT; ++mt_) {
          const unsigned char* wrow = wst + (mbase + mt_ * 32 + ln) * g::WST_ROWB + l0 * 2;
          bh[mt_] = as_bf16x8(*reinterpret_cast<const uintx4*>(wrow));
          bm[mt_] = as_bf16x8(*reinterpret_cast<const uintx4*>(wrow + g::WST_PLANEB));
        }
#pragma unroll
        for (int mt_ = 0; mt_ < MT; ++mt_) gt[gr * MT + mt_] = CAFEQ_MFMA_BF16(asl, bh[mt_], gt[gr * MT + mt_]);
#pragma unroll
        for (int mt_ = 0; mt_ < MT; ++mt_) gt[gr * MT + mt_] = CAFEQ_MFMA_BF16(ash, bm[mt_], gt[gr * MT + mt_]);
#pragma unroll
        for (int mt_ = 0; mt_ < MT; ++mt_) gt[gr * MT + mt_] = CAFEQ_MFMA_BF16(ash, bh[mt_], gt[gr * MT + mt_]);
      }
    }
    if (has_next) loader.finish();
    __syncthreads();   // the staging area is rewritten by the next macro-tile
    seg = nseg_;
    mis = nmis;
  }
  flush(cur_seg);
}

// grec[group][line] = the record of the group's first segment with the largest magnitude (ties: the lowest
// index wins, as inside a segment), its index moved from the segment to the group.  One thread per
// (group, line); rec is [segment][line] (one group per segment in that sweep).
__global__ __launch_bounds__(256) void combine_records_kernel(const float2* __restrict__ rec, int gspan, int L,
                                                               int64_t nlines, int64_t ngroups,
                                                               float2* __restrict__ grec,
                                                               const float2* __restrict__ rec_mm,
                                                               float2* __restrict__ grec_mm) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= ngroups * nlines) return;
  const int64_t gi = i / nlines, line = i - gi * nlines;
  float2 best = rec[(gi * gspan) * nlines + line];
  int bs = 0;
  for (int s = 1; s < gspan; ++s) {
    const float2 r = rec[(gi * gspan + s) * nlines + line];
    if (fabsf(r.x) > fabsf(best.x)) { best = r; bs = s; }
  }
  grec[i] = make_float2(best.x, __int_as_float(bs * L + __float_as_int(best.y)));
  if (rec_mm) {
    float2 mm = rec_mm[(gi * gspan) * nlines + line];
    for (int s = 1; s < gspan; ++s) {
      const float2 r = rec_mm[(gi * gspan + s) * nlines + line];
      mm.x = fminf(mm.x, r.x);
      mm.y = fmaxf(mm.y, r.y);
    }
    grec_mm[i] = mm;
  }
}

}  // namespace cafeq
