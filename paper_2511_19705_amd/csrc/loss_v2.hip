// Loss pass over PREPARED weights for 128 x 128 transform blocks (paper Sec. 4 / 4.1 / 4.2: transform,
// per-group absmax quantizer, inverse transform of the rounding error, l2 proxy, surrogate partials).
//
// The weights are constant over the tens of thousands of evaluations of a learning run, so
// cafeq_prepare_weights() stores them once in the form the matrix cores consume: per tile of 32 lines x
// 128 axis indices, two float16 parts (hi + lo of the line scaled by a power of two to [2^3, 2^4)) laid
// out so that one 16-byte load per lane is the B operand of one MFMA step -- the same 4 bytes per element
// as float32, no per-call splitting, every load a contiguous kilobyte per wave.  ||W||^2 and the per-line
// scale factors are stored beside them.
//
// Kernel shape.  One workgroup of eight waves per compute unit (two waves per SIMD).  The operand planes of
// the current block -- T and T^-1, float16 hi and lo parts each, 128 KB -- stay in LDS for as long as
// the workgroup works inside one segment, so they are fetched once per segment instead of once per
// macro-tile.  Each wave owns strips of 32 lines and alternates between a matrix phase
//   M(i) = inverse transform of strip i-1's error  +  forward transform of strip i
// and a vector phase
//   V(i) = quantizer epilogue of strip i (scale back, group absmax / arg-max, codes, error, records)
// with one workgroup barrier per phase; waves 4-7 run one phase behind waves 0-3, so that on every SIMD one
// wave feeds the matrix pipe while the other occupies the vector pipe (two independent workgroups drift
// into running the same phase at the same time and then share each pipe in turn).
//
// Arithmetic.  Forward: three float16 part products (hi.hi, hi.lo, lo.hi), float32 accumulation, exact
// scaling back by powers of two.  The scalings -- a line's weights below 2^4, a block's entries below 2^5 --
// bound every accumulator by 128 * 2^9 = 2^16, so the rounding error of the quantizer, at most half a step
// = absmax / (2 qmax) <= 2^15 in accumulator units, is a float16 number without any rescaling (the matrix
// cores take denormal float16 inputs exactly, so small entries lose nothing).  Inverse: the error E as ONE
// float16 part (round to nearest even: 2^-12 relative, zero mean) times T^-1 as hi + lo (2^-22 relative: a
// fixed operand's rounding would otherwise bias every element the same way).
#include "xform_core.hpp"

namespace cafeq {

namespace {

constexpr int kV2Waves = 8;
constexpr int kV2Threads = kV2Waves * 64;
constexpr int kV2MacroLines = kV2Waves * 32;
constexpr int kV2TileBytes = 32 * 128 * 4;            // one prepared tile: [8 steps][2 parts][64 lanes][16 B]
constexpr int kV2PlaneBytes = 4 * 2 * 128 * 64;        // one operand (T or T^-1) of one block: 64 KB
constexpr int kV2Lds = 2 * kV2PlaneBytes + kV2Waves * kHdrFloats * 4 + 64;

// REC: write the arg-max records (the gradient pass follows); OUT: write scales and / or codes
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
// (x0, x1) -> packed float16 pair, round to nearest even (one v_cvt_pk_f16_f32), x0 in the low half
__device__ __forceinline__ uint32_t pack_f16(float x0, float x1) {
  floatx2 v = {x0, x1};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, halfx2));
}

// bidx: the workgroup's index among the p.nwg workgroups that share the matrix
template <int G, int AXIS, bool REC, bool OUT>
__device__ __forceinline__ void loss_v2_body(const CoreParams& p, const unsigned bidx) {
  constexpr int L = 128, KT = 4, NGRP = L / G, RPG = G / 2;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* lfw = smem;                      // forward planes [4 stages][hi, lo][128 rows][64 B]
  unsigned char* liv = smem + kV2PlaneBytes;      // inverse planes [4 stages][hi, lo][128 rows][64 B]
  float* hred = reinterpret_cast<float*>(smem + 2 * kV2PlaneBytes);   // [8 waves][kHdrFloats]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;                      // phase group: waves 4-7 run one phase behind (waves i and i + 4 share a SIMD)
  const int ln = lane & 31, h = lane >> 5;

  int64_t w = bidx;
  if ((p.nwg & 7) == 0) w = int64_t(bidx & 7) * (p.nwg >> 3) + (bidx >> 3);
  const int64_t mt0 = chunk_begin(w, p.n_mt, p.nwg), mt1 = chunk_begin(w + 1, p.n_mt, p.nwg);
  if (mt0 >= mt1) return;
  const int mt_per_seg = int(p.mt_per_seg);       // macro-tiles of 256 lines per segment
  const int64_t nlp = int64_t(mt_per_seg) * kV2MacroLines;
  const bool lse_on = p.loss_kind == kLossLse;
  const int swz = (ln >> 2) & 3;
  const int aoff0 = ln * 64 + ((h ^ swz) << 4), aoff1 = ln * 64 + (((2 + h) ^ swz) << 4);
  bool wsq_pending = w == 0;

  // per-lane running sums of the current segment
  float s_l2 = 0.f, s_errz = 0.f, s_sur = 0.f, m_ref = -INFINITY;
  float s_va2[NGRP];
#pragma unroll
  for (int i = 0; i < NGRP; ++i) s_va2[i] = 0.f;

  // Prepared B operands of the strip the next forward phase transforms, and that strip's line scale factor.
  // They are requested a whole vector phase ahead of their use (at the start of the vector phase of the strip
  // before, across run boundaries too), so that their latency never reaches the matrix pipe: requested at the
  // start of the matrix phase they had only the inverse transform (about a microsecond) to arrive in.
  uintx4 wq[16];
  float lsc_nx = 0.f;
  auto request_strip = [&](int sg, int64_t strip) {   // strip: the wave's strip inside segment sg
    lsc_nx = p.prep_lscale[int64_t(sg) * nlp + strip * 32 + ln];
    const unsigned char* tp = p.prep_planes + (int64_t(sg) * (nlp / 32) + strip) * kV2TileBytes + lane * 16;
#pragma unroll
    for (int i = 0; i < 16; ++i) wq[i] = *reinterpret_cast<const uintx4*>(tp + i * 1024);
  };
  // (The variants that write codes or scales keep their requests at the start of the matrix phase: their vector
  // phase has no registers to hold a strip in flight.)
  constexpr bool EARLY = !OUT;
  // (16-byte code stores need the code matrix aligned to 16 bytes; its row length is a multiple of 128)
  const bool wide_codes = OUT && (reinterpret_cast<uintptr_t>(p.codes) & 15) == 0;
  if constexpr (EARLY) {
    const int sg = int(mt0 / mt_per_seg);
    request_strip(sg, (mt0 - int64_t(sg) * mt_per_seg) * kV2Waves + wave);
  }

  for (int64_t mt = mt0; mt < mt1;) {
    const int seg = int(mt / mt_per_seg);
    const int mis0 = int(mt - int64_t(seg) * mt_per_seg);
    const int n = int(mt1 - mt < int64_t(mt_per_seg - mis0) ? mt1 - mt : int64_t(mt_per_seg - mis0));
    const int bid = p.rep != 1 ? seg / p.rep : seg;   // (rep is 1 on the column axis)

    // ---- the block's operand planes into LDS (the previous segment's readers are past flush's barriers)
    {
      const uintx4* gf = reinterpret_cast<const uintx4*>(reinterpret_cast<const unsigned char*>(p.Afwd) + int64_t(bid) * kV2PlaneBytes);
      const uintx4* gi = reinterpret_cast<const uintx4*>(reinterpret_cast<const unsigned char*>(p.Ainv) + int64_t(bid) * kV2PlaneBytes);
      uintx4 tf[8], ti[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { tf[i] = gf[i * kV2Threads + tid]; ti[i] = gi[i * kV2Threads + tid]; }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        reinterpret_cast<uintx4*>(lfw)[i * kV2Threads + tid] = tf[i];
        reinterpret_cast<uintx4*>(liv)[i * kV2Threads + tid] = ti[i];
      }
    }
    const float fsc = p.fscale[bid];
    const float fsi = p.fscale_inv[bid];
    __syncthreads();

    float usc = 0.f;          // the factor back to the units of Z for the strip in the accumulators
    float usc2_prev = 0.f;    // its square for the strip whose error the next inverse phase transforms
    floatx16 acc[KT];
    uint32_t ebf[L / 4];      // the error as packed float16 (accumulator units): B operands of the inverse phase
    // the strip after strip m of this run: the run's next one, else the first of the next run (the next segment),
    // else -- the range ends here -- strip m once more (an unconditional request keeps the wait counts exact)
    const bool more_runs = mt + n < mt1;
    auto request_next = [&](int m) {
      int sg = seg;
      int64_t strip = int64_t(mis0 + m + 1) * kV2Waves + wave;
      if (m + 1 == n) {
        if (more_runs) { sg = seg + 1; strip = wave; }
        else strip -= kV2Waves;
      }
      request_strip(sg, strip);
    };

    // Both contractions walk the output tiles one after the other (tile t: 32 outputs, its accumulator a
    // chain of MFMAs over the eight steps of 16 inputs), so that only a few operand registers are live: the
    // A operands (transform tiles from LDS) are requested two steps ahead into a rotating set of three, the
    // B operands are the lane's own registers.  Scheduling barriers pin the issue order per step: the LDS reads
    // of step + 2, then the step's MFMAs and vector work (the compiler would otherwise sink each read to just
    // before its use and wait for it there).
    //
    // matrix phase, second half: forward transform of the strip in wq
    auto forward = [&]() {
      const unsigned char* b0 = lfw + aoff0;
      const unsigned char* b1 = lfw + aoff1;
      auto frag = [&](int i, int pl) {   // i = 8 t + c
        const int t = i >> 3, c = i & 7;
        return *reinterpret_cast<const uintx4*>(((c & 1) ? b1 : b0) + (c >> 1) * (2 * 128 * 64) + pl * (128 * 64) + t * (32 * 64));
      };
      uintx4 fh[3], fl[3];
      fh[0] = frag(0, 0); fl[0] = frag(0, 1);
      fh[1] = frag(1, 0); fl[1] = frag(1, 1);
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        floatx16 a;
#pragma unroll
        for (int v = 0; v < 16; ++v) a[v] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int i = 8 * t + c;
          if (i + 2 < 8 * KT) { fh[(i + 2) % 3] = frag(i + 2, 0); fl[(i + 2) % 3] = frag(i + 2, 1); }
          __builtin_amdgcn_sched_barrier(0);     // the reads of step + 2 are issued before this step's products
          const halfx8 xh = as_halfx8(fh[i % 3]), xl = as_halfx8(fl[i % 3]);
          const halfx8 vbh = as_halfx8(wq[2 * c]), vbl = as_halfx8(wq[2 * c + 1]);
          a = CAFEQ_MFMA_F16(xl, vbh, a);
          a = CAFEQ_MFMA_F16(xh, vbl, a);
          a = CAFEQ_MFMA_F16(xh, vbh, a);
          __builtin_amdgcn_sched_barrier(0);
        }
        acc[t] = a;
      }
    };
    // matrix phase, first half: D^T = Ainv . E^T for the strip whose error is in ebf, and the sum of its squares
    // (a tile's sum runs in the shadow of the next tile's products)
    auto inverse = [&](float usc2_strip) {
      float l2 = 0.f;               // in the units of the strip's accumulators
      const unsigned char* b0 = liv + aoff0;
      const unsigned char* b1 = liv + aoff1;
      auto frag = [&](int i, int pl) {
        const int t = i >> 3, c = i & 7;
        return *reinterpret_cast<const uintx4*>(((c & 1) ? b1 : b0) + (c >> 1) * (2 * 128 * 64) + pl * (128 * 64) + t * (32 * 64));
      };
      // (two products per step cover only 64 cycles of matrix time, so the reads run four steps ahead)
      constexpr int DI = 4;
      uintx4 fh[DI + 1], fm[DI + 1];
#pragma unroll
      for (int i = 0; i < DI; ++i) { fh[i] = frag(i, 0); fm[i] = frag(i, 1); }
      floatx16 dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) dp[v] = 0.f;
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        floatx16 a;
#pragma unroll
        for (int v = 0; v < 16; ++v) a[v] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int i = 8 * t + c;
          if (i + DI < 8 * KT) { fh[(i + DI) % (DI + 1)] = frag(i + DI, 0); fm[(i + DI) % (DI + 1)] = frag(i + DI, 1); }
          __builtin_amdgcn_sched_barrier(0);
          const halfx8 xh = as_halfx8(fh[i % (DI + 1)]), xm = as_halfx8(fm[i % (DI + 1)]);
          const halfx8 ve = as_halfx8(ebf[4 * c], ebf[4 * c + 1], ebf[4 * c + 2], ebf[4 * c + 3]);
          a = CAFEQ_MFMA_F16(xm, ve, a);
          a = CAFEQ_MFMA_F16(xh, ve, a);
          l2 = fmaf(dp[2 * c], dp[2 * c], l2);            // previous tile (zeros for the first)
          l2 = fmaf(dp[2 * c + 1], dp[2 * c + 1], l2);
          __builtin_amdgcn_sched_barrier(0);
        }
        dp = a;
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) l2 = fmaf(dp[v], dp[v], l2);
      s_l2 = fmaf(l2, usc2_strip, s_l2);
    };
    // vector phase: the quantizer on strip m (accumulators -> error).  The accumulators hold Z / usc with usc a
    // power of two per line, and everything up to the error stays in those units: absmax, reciprocal, codes and
    // error scale exactly (q = rint(z' * fl(qmax / a')) is the recipe's rint(z * fl(qmax / a)) bit for bit), so
    // the 64 multiplications back to the units of Z are replaced by a few per group and per strip.  (The two
    // differ only where a group's absmax or scale would be a denormal float32, below 1e-37.)
    auto epilogue = [&](int m) {
      const int64_t line = int64_t(mis0 + m) * kV2MacroLines + wave * 32 + ln;
      const bool valid = line < p.nlines;
      const int64_t ax0 = int64_t(seg) * L;
      const float usc2 = usc * usc;
      const float dsc = usc * fsi;  // inverse-transformed error: accumulator units -> units of W
      float e2 = 0.f;               // sum of squared errors of this strip in accumulator units
#pragma unroll
      for (int gi = 0; gi < NGRP; ++gi) {
        float zs = 0.f;
        int jf = 0;
        if constexpr (REC) {
          // signed value at the arg-max and its index (without the lane-half term): an immediate per register
#pragma unroll
          for (int f = gi * RPG; f < (gi + 1) * RPG; ++f) {
            const float z = acc[f / 16][f % 16];
            if (fabsf(z) > fabsf(zs)) { zs = z; jf = 8 * (f / 4) + (f % 4); }
          }
        } else {
          float a0 = 0.f;
#pragma unroll
          for (int f = gi * RPG; f < (gi + 1) * RPG; f += 2)
            a0 = fmaxf(fmaxf(fabsf(acc[f / 16][f % 16]), fabsf(acc[(f + 1) / 16][(f + 1) % 16])), a0);
          zs = a0;
        }
        float as = fabsf(zs);       // absmax in accumulator units
        {
          const float oz = __shfl_xor(zs, 32);
          const float oa = fabsf(oz);
          if constexpr (REC) {
            int j = jf + 4 * h;
            const int oj = __shfl_xor(j, 32);
            if (oa > as || (oa == as && oj < j)) { as = oa; zs = oz; j = oj; }
            if (valid && h == 0)
              p.rec[(int64_t(seg) * NGRP + gi) * p.nlines + line] = make_float2(zs * usc, __int_as_float(j - gi * G));
          } else {
            as = fmaxf(as, oa);
          }
        }
        const float a = as * usc;   // exact
        const float inv = grid_inv(as, p.grid.qmax);
        const float s = grid_scale(as, p.grid.qmax);
        if (OUT && p.scales && valid && h == 0) {
          const int64_t gidx = ax0 / G + gi;
          const float st = grid_scale(a, p.grid.qmax);
          if (AXIS == CAFEQ_AXIS_COL) p.scales[line * (p.cols / G) + gidx] = st;
          else p.scales[gidx * p.cols + line] = st;
        }
#pragma unroll
        for (int f2 = gi * RPG / 2; f2 < (gi + 1) * RPG / 2; ++f2) {
          float er[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int f = 2 * f2 + e;
            const float z = acc[f / 16][f % 16];
            // |z * inv| <= qmax (1 + 2^-23), so the rounded value is already inside the grid: no clamp.
            // The error is taken with one rounding, q s - z (the recipe's fl(q s) - z differs by 2^-24 |q s|,
            // at most 2e-6 of the error's own size on grids of up to 4 bits).
            const float q = __builtin_rintf(__fmul_rn(z, inv));
            er[e] = fmaf(q, s, -z);
            if constexpr (OUT) acc[f / 16][f % 16] = q;            // kept for the optional code output
          }
          ebf[f2] = pack_f16(er[0], er[1]);
          // the sum of squared errors from the packed pair (one dot-product instruction per pair; the float16
          // rounding of an error is 2^-12 relative and random in sign, far below the sum's budget)
          e2 = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2, ebf[f2]), __builtin_bit_cast(halfx2, ebf[f2]), e2, false);
        }
        const float a2 = a * a;
        if (h == 0) s_va2[gi] += a2;
        if (!lse_on && h == 0) s_sur = fmaf(a2, p.rG[seg * NGRP + gi], s_sur);
        if (lse_on) {
          // exponentials relative to this wave's running reference
          const float am = valid ? a : 0.f;
          const float nm = fmaxf(cluster_allmax<64>(am), m_ref);
          if (nm > m_ref) {
            s_sur *= __expf(p.lse_t * (m_ref - nm));   // 0 on the first group
            m_ref = nm;
          }
          if (valid && h == 0) s_sur += __expf(p.lse_t * (a - m_ref));
        }
      }
      s_errz = fmaf(e2, usc2, s_errz);
      if (OUT && AXIS == CAFEQ_AXIS_COL && L == 128 && p.codes && wide_codes) {
        // A line's 128 codes are spread over its two lanes in alternating 4-byte words (word f4 of lane half h:
        // codes 8 f4 + 4 h ..).  Swapping the upper lanes' word a with the lower lanes' word a + 8 leaves codes
        // 0..63 in the lower lane and 64..127 in the upper one: four 16-byte stores per lane instead of sixteen
        // 4-byte ones.
        uint32_t wd[16];
#pragma unroll
        for (int f4 = 0; f4 < 16; ++f4) {
          const int f = 4 * f4;
          wd[f4] = pack4(acc[f / 16][f % 16], acc[f / 16][f % 16 + 1], acc[f / 16][f % 16 + 2], acc[f / 16][f % 16 + 3]);
        }
#pragma unroll
        for (int a = 0; a < 8; ++a) {
          const auto r = __builtin_amdgcn_permlane32_swap(wd[a], wd[a + 8], false, false);
          wd[a] = r[0];
          wd[a + 8] = r[1];
        }
        if (valid) {
          int8_t* dst = p.codes + line * p.cols + ax0 + 64 * h;
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            uintx4 v;
            v[0] = wd[2 * m]; v[1] = wd[2 * m + 8]; v[2] = wd[2 * m + 1]; v[3] = wd[2 * m + 9];
            *reinterpret_cast<uintx4*>(dst + 16 * m) = v;
          }
        }
      } else if (OUT && p.codes && valid) {
#pragma unroll
        for (int f4 = 0; f4 < L / 8; ++f4) {
          const int f = 4 * f4;
          const uint32_t pk = pack4(acc[f / 16][f % 16], acc[f / 16][f % 16 + 1], acc[f / 16][f % 16 + 2], acc[f / 16][f % 16 + 3]);
          const int j0 = 8 * f4 + 4 * h;
          if (AXIS == CAFEQ_AXIS_COL) {
            *reinterpret_cast<uint32_t*>(p.codes + line * p.cols + ax0 + j0) = pk;
          } else {
            int8_t* rowp = p.codes + (ax0 + j0) * p.cols + line;
#pragma unroll
            for (int e = 0; e < 4; ++e) rowp[int64_t(e) * p.cols] = int8_t(pk >> (8 * e));
          }
        }
      }
      return dsc * dsc;
    };

    // ---- the phases of this run of n macro-tiles: strip m = matrix phase (inverse transform of strip m-1,
    // forward transform of strip m), barrier, vector phase (epilogue of strip m), barrier; one more matrix
    // phase for the last strip's inverse transform.  Group 1 runs one phase behind group 0: it waits one barrier
    // before its first phase, group 0 one after its last.  The first and the last phase are written out
    // separately so that inside the loop every register array is defined and consumed in the same iteration.
    //
    // Phase fences.  The compiler may move register-only work across a barrier; the empty asm statements take a
    // phase's results as in-out operands, so that everything that produces them stays before the barrier and
    // everything that consumes them after it (the scale factor included: the wait for its load belongs to the
    // matrix phase, so that the vector phase never waits on the memory counter).
    auto fence_m = [&]() {
      asm volatile("" : "+v"(usc), "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
      __builtin_amdgcn_s_barrier();
    };
    auto fence_v = [&]() {
      asm volatile("" : "+v"(ebf[0]), "+v"(ebf[1]), "+v"(ebf[2]), "+v"(ebf[3]), "+v"(ebf[4]), "+v"(ebf[5]), "+v"(ebf[6]),
                   "+v"(ebf[7]), "+v"(ebf[8]), "+v"(ebf[9]), "+v"(ebf[10]), "+v"(ebf[11]), "+v"(ebf[12]), "+v"(ebf[13]),
                   "+v"(ebf[14]), "+v"(ebf[15]));
      asm volatile("" : "+v"(ebf[16]), "+v"(ebf[17]), "+v"(ebf[18]), "+v"(ebf[19]), "+v"(ebf[20]), "+v"(ebf[21]),
                   "+v"(ebf[22]), "+v"(ebf[23]), "+v"(ebf[24]), "+v"(ebf[25]), "+v"(ebf[26]), "+v"(ebf[27]), "+v"(ebf[28]),
                   "+v"(ebf[29]), "+v"(ebf[30]), "+v"(ebf[31]), "+v"(usc2_prev));
      __builtin_amdgcn_s_barrier();
    };
    if (grp == 1) __builtin_amdgcn_s_barrier();
    {
      if constexpr (!EARLY) request_strip(seg, int64_t(mis0) * kV2Waves + wave);
      forward();
      usc = lsc_nx * fsc;
      fence_m();
      if constexpr (EARLY) request_next(0);
      usc2_prev = epilogue(0);
      fence_v();
    }
    for (int m = 1; m < n; ++m) {
      // The matrix phase wins the issue arbitration on its SIMD: its MFMAs go out as soon as the matrix pipe is
      // free and the other wave's vector phase fills the issue slots in between (at equal priority the vector
      // stream crowds out the first part of this phase and then leaves the rest of it without company).
      if constexpr (!EARLY) request_strip(seg, int64_t(mis0 + m) * kV2Waves + wave);
      __builtin_amdgcn_s_setprio(3);
      inverse(usc2_prev);
      forward();
      __builtin_amdgcn_s_setprio(0);
      usc = lsc_nx * fsc;
      fence_m();
      if constexpr (EARLY) request_next(m);
      usc2_prev = epilogue(m);
      fence_v();
    }
    inverse(usc2_prev);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_s_barrier();
    if (grp == 0) __builtin_amdgcn_s_barrier();

    // ---- publish this (workgroup, segment) partial: per-lane sums -> waves -> workgroup
    {
      const int64_t slot = w + seg;
      float vals[kHdrVa2 + NGRP];
      vals[kHdrL2] = s_l2; vals[kHdrErrZ] = s_errz; vals[kHdrWsq] = 0.f; vals[kHdrSur] = s_sur;
      vals[kHdrMref] = 0.f; vals[5] = 0.f; vals[6] = 0.f; vals[7] = 0.f;
#pragma unroll
      for (int i = 0; i < NGRP; ++i) vals[kHdrVa2 + i] = s_va2[i];
#pragma unroll
      for (int i = 0; i < kHdrVa2 + NGRP; ++i) {
        const float t = wave_sum(vals[i]);
        if (lane == 0) hred[wave * kHdrFloats + i] = t;
      }
      if (lane == 0) hred[wave * kHdrFloats + kHdrMref] = m_ref;
      __syncthreads();
      if (tid < kHdrVa2 + NGRP) {
        float t = 0.f;
        if (tid == kHdrMref || (tid == kHdrSur && lse_on)) {
          // waves keep their own references: rescale their sums of exponentials to the largest
          float mm = -INFINITY;
#pragma unroll
          for (int ww = 0; ww < kV2Waves; ++ww) mm = fmaxf(mm, hred[ww * kHdrFloats + kHdrMref]);
          if (tid == kHdrMref) {
            t = mm;
          } else {
#pragma unroll
            for (int ww = 0; ww < kV2Waves; ++ww) {
              const float sw = hred[ww * kHdrFloats + kHdrSur];
              if (sw > 0.f) t += sw * __expf(p.lse_t * (hred[ww * kHdrFloats + kHdrMref] - mm));
            }
          }
        } else {
#pragma unroll
          for (int ww = 0; ww < kV2Waves; ++ww) t += hred[ww * kHdrFloats + tid];
        }
        if (tid == kHdrWsq && wsq_pending) t = *p.prep_wsq;
        p.slot_hdr[slot * kHdrFloats + tid] = t;
      }
      wsq_pending = false;
      __syncthreads();
      s_l2 = s_errz = s_sur = 0.f;
      m_ref = -INFINITY;
#pragma unroll
      for (int i = 0; i < NGRP; ++i) s_va2[i] = 0.f;
    }
    mt += n;
  }
}

template <int G, int AXIS, bool REC, bool OUT>
__global__ __launch_bounds__(kV2Threads, 1) void loss_v2_kernel(const CoreParams p) {
  loss_v2_body<G, AXIS, REC, OUT>(p, blockIdx.x);
}

// Both members of a pair in one launch (no codes or scales requested): the first pa.nwg workgroups take member
// A, the others member B.  With one workgroup per compute unit in total, half of the chip streams each member
// and the ranges of the two members end together -- one kernel tail instead of two.
template <int G, bool REC>
__global__ __launch_bounds__(kV2Threads, 1) void loss_v2_pair_kernel(const CoreParams pa, const CoreParams pb) {
  if (blockIdx.x < unsigned(pa.nwg)) loss_v2_body<G, CAFEQ_AXIS_COL, REC, false>(pa, blockIdx.x);
  else loss_v2_body<G, CAFEQ_AXIS_ROW, REC, false>(pb, blockIdx.x - unsigned(pa.nwg));
}

// ---------------------------------------------------------------------------------------------------
// preparation: one workgroup per tile of 32 lines x 128 axis indices
// ---------------------------------------------------------------------------------------------------
struct PrepArgs {
  const void* W; int dtype; int64_t rows, cols, ld; int axis;
  int64_t nlines, nlp; int nseg;
  unsigned char* planes; float* lscale; double* partial;
};

__global__ __launch_bounds__(256) void prepare_tiles_kernel(const PrepArgs a) {
  __shared__ float tile[32][129];
  __shared__ double red[4];
  const int64_t nstrip = a.nlp / 32;
  const int64_t tix = blockIdx.x;
  const int seg = int(tix / nstrip);
  const int64_t strip = tix - int64_t(seg) * nstrip;
  const int t = threadIdx.x;
  for (int r = 0; r < 16; ++r) {
    const int idx = r * 256 + t;
    int li, m;
    if (a.axis == CAFEQ_AXIS_COL) { li = idx >> 7; m = idx & 127; } else { m = idx >> 5; li = idx & 31; }
    const int64_t line = strip * 32 + li, ax = int64_t(seg) * 128 + m;
    float v = 0.f;
    if (line < a.nlines) {
      const int64_t off = a.axis == CAFEQ_AXIS_COL ? line * a.ld + ax : ax * a.ld + line;
      v = a.dtype == CAFEQ_F32 ? static_cast<const float*>(a.W)[off]
                               : bf16_bits_to_f32(static_cast<const uint16_t*>(a.W)[off]);
    }
    tile[li][m] = v;
  }
  __syncthreads();
  const int li = t >> 3, c = t & 7;
  float x[16];
  float mx = 0.f;
  double sq = 0;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    x[e] = tile[li][16 * c + e];
    mx = fmaxf(mx, fabsf(x[e]));
    sq += double(x[e]) * x[e];
  }
  mx = fmaxf(mx, __shfl_xor(mx, 1));
  mx = fmaxf(mx, __shfl_xor(mx, 2));
  mx = fmaxf(mx, __shfl_xor(mx, 4));
  int ex = int(__float_as_uint(mx) >> 23);
  ex = ex < 32 ? 32 : (ex > 254 ? 254 : ex);        // lines of (almost) zeros: any scale will do
  const float wsc = __uint_as_float(uint32_t(257 - ex) << 23);          // 2^(3 - (ex - 127)): largest magnitude in [2^3, 2^4)
  if (c == 0) a.lscale[int64_t(seg) * a.nlp + strip * 32 + li] = __uint_as_float(uint32_t(ex - 3) << 23);
  unsigned char* tp = a.planes + tix * int64_t(kV2TileBytes) + c * 2048;
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      uint32_t hb[2], lb[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float y = x[8 * hh + 2 * e2 + u] * wsc;
        const _Float16 p0 = _Float16(y);
        const _Float16 p1 = _Float16(y - float(p0));
        hb[u] = __builtin_bit_cast(uint16_t, p0);
        lb[u] = __builtin_bit_cast(uint16_t, p1);
      }
      hi[e2] = hb[0] | (hb[1] << 16);
      lo[e2] = lb[0] | (lb[1] << 16);
    }
    *reinterpret_cast<uint4*>(tp + (hh * 32 + li) * 16) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    *reinterpret_cast<uint4*>(tp + 1024 + (hh * 32 + li) * 16) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
  }
  sq = wave_sum(sq);
  if ((t & 63) == 0) red[t >> 6] = sq;
  __syncthreads();
  if (t == 0) a.partial[tix] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void prepare_sum_kernel(const double* __restrict__ partial, int64_t n,
                                                           float* __restrict__ out) {
  __shared__ double red[256];
  double t = 0;
  for (int64_t i = threadIdx.x; i < n; i += 256) t += partial[i];
  red[threadIdx.x] = t;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = float(red[0]);
}

template <int G, int AXIS, bool REC, bool OUT>
int launch_v2_v(const CoreParams& p, hipStream_t st) {
  auto kern = loss_v2_kernel<G, AXIS, REC, OUT>;
  static std::atomic<bool> attr_set{false};   // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return CAFEQ_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(unsigned(p.nwg)), dim3(kV2Threads), kV2Lds, st, p);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
template <int G, int AXIS>
int launch_v2_t(const CoreParams& p, hipStream_t st) {
  if (p.codes || p.scales)
    return p.rec ? launch_v2_v<G, AXIS, true, true>(p, st) : launch_v2_v<G, AXIS, false, true>(p, st);
  return p.rec ? launch_v2_v<G, AXIS, true, false>(p, st) : launch_v2_v<G, AXIS, false, false>(p, st);
}

}  // namespace

PreparedLayout prepared_layout(int64_t nlines, int64_t naxis) {
  PreparedLayout l;
  l.nlp = (nlines + kV2MacroLines - 1) / kV2MacroLines * kV2MacroLines;
  l.nseg = naxis / 128;
  l.ntiles = l.nseg * (l.nlp / 32);
  l.off_lscale = 256;
  l.off_planes = align_up(l.off_lscale + size_t(l.nseg) * l.nlp * sizeof(float), 256);
  l.off_partial = l.off_planes + size_t(l.ntiles) * kV2TileBytes;
  l.off_gtiles = align_up(l.off_partial + size_t(l.ntiles) * sizeof(double), 256);
  l.bytes = align_up(l.off_gtiles + prepared_gtiles_bytes(nlines, naxis), 256);
  return l;
}

int launch_prepare(const cafeq_mat* W, int axis, void* prepared, hipStream_t st) {
  const bool col = axis == CAFEQ_AXIS_COL;
  const int64_t nlines = col ? W->rows : W->cols, naxis = col ? W->cols : W->rows;
  if (naxis % 128 != 0) return CAFEQ_ERR_BAD_SHAPE;
  const PreparedLayout l = prepared_layout(nlines, naxis);
  unsigned char* base = static_cast<unsigned char*>(prepared);
  PrepArgs a;
  a.W = W->data; a.dtype = W->dtype; a.rows = W->rows; a.cols = W->cols; a.ld = W->ld; a.axis = axis;
  a.nlines = nlines; a.nlp = l.nlp; a.nseg = int(l.nseg);
  a.planes = base + l.off_planes; a.lscale = reinterpret_cast<float*>(base + l.off_lscale);
  a.partial = reinterpret_cast<double*>(base + l.off_partial);
  hipLaunchKernelGGL(prepare_tiles_kernel, dim3(unsigned(l.ntiles)), dim3(256), 0, st, a);
  CAFEQ_CHECK_LAUNCH();
  hipLaunchKernelGGL(prepare_sum_kernel, dim3(1), dim3(256), 0, st, a.partial, l.ntiles, reinterpret_cast<float*>(base));
  CAFEQ_CHECK_LAUNCH();
  return launch_prepare_gtiles(W, axis, base + l.off_gtiles, st);
}

namespace {
template <int G, bool REC>
int launch_v2_pair_v(const CoreParams& pa, const CoreParams& pb, hipStream_t st) {
  auto kern = loss_v2_pair_kernel<G, REC>;
  static std::atomic<bool> attr_set{false};   // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024) != hipSuccess)
      return CAFEQ_ERR_LAUNCH;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(unsigned(pa.nwg + pb.nwg)), dim3(kV2Threads), kV2Lds, st, pa, pb);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
}  // namespace

// Both members of a pair (member A on its columns, member B on its rows) in one launch; same group length and
// the same choice of records for both, no codes or scales.
int launch_loss_v2_pair(int G, const CoreParams& pa, const CoreParams& pb, hipStream_t st) {
  for (const CoreParams* p : {&pa, &pb})
    if (!p->prep_planes || !p->prep_lscale || !p->prep_wsq || !p->fscale || !p->fscale_inv || !p->slot_hdr || p->codes ||
        p->scales)
      return CAFEQ_ERR_INVALID_ARG;
  if ((pa.rec != nullptr) != (pb.rec != nullptr)) return CAFEQ_ERR_INVALID_ARG;
  const bool rec = pa.rec != nullptr;
  switch (G) {
    case 32: return rec ? launch_v2_pair_v<32, true>(pa, pb, st) : launch_v2_pair_v<32, false>(pa, pb, st);
    case 64: return rec ? launch_v2_pair_v<64, true>(pa, pb, st) : launch_v2_pair_v<64, false>(pa, pb, st);
    case 128: return rec ? launch_v2_pair_v<128, true>(pa, pb, st) : launch_v2_pair_v<128, false>(pa, pb, st);
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
}

int launch_loss_v2(int G, int axis, const CoreParams& p, hipStream_t st) {
  if (!p.prep_planes || !p.prep_lscale || !p.prep_wsq || !p.fscale || !p.fscale_inv || !p.slot_hdr) return CAFEQ_ERR_INVALID_ARG;
  const bool col = axis == CAFEQ_AXIS_COL;
  switch (G) {
    case 32: return col ? launch_v2_t<32, CAFEQ_AXIS_COL>(p, st) : launch_v2_t<32, CAFEQ_AXIS_ROW>(p, st);
    case 64: return col ? launch_v2_t<64, CAFEQ_AXIS_COL>(p, st) : launch_v2_t<64, CAFEQ_AXIS_ROW>(p, st);
    case 128: return col ? launch_v2_t<128, CAFEQ_AXIS_COL>(p, st) : launch_v2_t<128, CAFEQ_AXIS_ROW>(p, st);
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
}

}  // namespace cafeq
