// Kernels of the adaptive-rounding step (paper Sec. 5, Alg. 1) in transformed coordinates.
//
// Alg. 1 alternates  W2^ <- Q(pinv(W1^) W1 W2)  and  W1^ <- Q(W1 W2 pinv(W2^)).  Per head the
// pseudoinverse of a full-column-rank (resp. full-row-rank) quantized block is formed from
// k x k normal equations.  With Xq the dequantized codes and E = Xq - X the current rounding
// error, both lines have the same shape:
//     S = Gram(Xq, Xq),  R = Gram(Xq, E),   C = I - S^-1 R
// where Gram(X, Y)[a][b] = sum_t X[t][a] Y[t][b]; t runs over the rows of U (line 3) or over
// the columns of the head's row-blocks of V (line 4), a and b over the k indices of the head.
// Line 3 quantizes C . V_q, line 4 quantizes U_b . C^T (the fused core is handed C as the
// [out][in] operand either way).  Working with E instead of X keeps the float32 Gram sums at
// the scale of the correction, not of the identity it is subtracted from.
//
//   gram_pair_kernel : fp32 MFMA (v_mfma_f32_32x32x2_f32), one workgroup per (head, 32-row
//                      output stripe, chunk of the contraction range); codes are dequantized
//                      on the fly; chunk partials are written out, not atomically added.
//   gram_pair16_kernel : the same pair for heads of 128 and 256 on the 16-bit matrix pipe, operands
//                      split exactly into three bfloat16 parts.
//   gj_panel_kernel  : sums the chunk partials of S in float64 and inverts it by register-
//                      resident Gauss-Jordan elimination with partial pivoting; also serves
//                      cafeq_block_inverse.  C = I - S^-1 R follows as a batched product.
//   gj_spd256_kernel : the inversion of S for heads of 256 as a block elimination whose products
//                      run on the 16-bit matrix pipe.
#include <atomic>
#include <type_traits>

#include "xform_core.hpp"

namespace cafeq {

namespace {

struct GramArgs {
  const float* X;        // original (transformed) matrix, float32 dense
  const int8_t* codes;   // its current codes
  const float* scales;   // its current scales
  int64_t rows, cols;
  int K, G, rep;
  int64_t tlen;          // contraction length per row-block (rows of U / columns of V)
  int64_t chunk;         // contraction elements per workgroup (multiple of 16)
  int nchunk;            // chunks per row-block
  float* partial;        // [nb][rep*nchunk][2 or 3][K][K]: Gram(Xq,Xq), Gram(Xq,E) and, TRIPLE, Gram(E,E)
};

// AXIS == COL: t = row i, free index = column;  AXIS == ROW: t = column c, free index = row.
// One workgroup per (head, 32-row output stripe jt1, chunk of the contraction range).  Per step
// of 16 contraction indices the workgroup loads the head's 16 x K slab of codes, scales and
// originals with wide coalesced loads, dequantizes it ONCE (Xq and E = Xq - X) into LDS laid out
// [t][free index], and every wave feeds its MFMAs from there: A = Xq[t][stripe columns] (shared
// by the waves), B = Xq / E [t][its output tiles].  The next slab's loads are in flight while
// the matrix cores work on the current one.
template <int AXIS, int K, bool TRIPLE>
__global__ __launch_bounds__(256) void gram_pair_kernel(const GramArgs a) {
  // row stride of the LDS slab: 16-byte aligned rows for the vector stores of the column case;
  // K + 2 for the row case, whose transposing scalar stores then spread over all banks
  constexpr int KT = K / 32, LD = AXIS == CAFEQ_AXIS_COL ? K + 4 : K + 2;
  __shared__ __align__(16) float qs[16 * LD];
  __shared__ __align__(16) float es[16 * LD];
  const int b = blockIdx.x, jt1 = blockIdx.y;
  const int z = blockIdx.z;                      // (row-block within head, chunk)
  const int qi = z / a.nchunk, ch = z % a.nchunk;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, h = lane >> 5;
  const int64_t t0 = int64_t(ch) * a.chunk;
  const int64_t t1 = t0 + a.chunk < a.tlen ? t0 + a.chunk : a.tlen;
  // free-index origin of this head / row-block
  const int64_t f0 = AXIS == CAFEQ_AXIS_COL ? int64_t(b) * K : (int64_t(b) * a.rep + qi) * K;
  const int64_t C = a.cols;

  // output tiles of this wave: jt2 = wave + 4u, u < NU; for K < 128 the waves beyond KT have none.  NU is a
  // compile-time count so that the accumulators stay where the matrix instructions want them.
  constexpr int NU = (KT + 3) / 4;
  const bool active = KT >= 4 || wave < KT;   // known at compile time for K >= 128: no branch around the MFMAs
  floatx16 accS[NU], accR[NU], accT[TRIPLE ? NU : 1];
#pragma unroll
  for (int u = 0; u < NU; ++u)
#pragma unroll
    for (int v = 0; v < 16; ++v) { accS[u][v] = 0.f; accR[u][v] = 0.f; accT[TRIPLE ? u : 0][v] = 0.f; }

  // ---- loader roles.  COL: thread -> (t = l / (K/EPT), EPT/4 chunks of four columns, the chunks of the
  // K/EPT threads of a row interleaved so that their 16-byte LDS stores fall into distinct banks);
  // ROW: NP passes of 64 rows, thread -> (row = pass*64 + l/4, four consecutive t = 4*(l%4) ..)
  constexpr int EPT = K >= 64 ? K / 16 : 4;          // COL: columns per thread
  constexpr int NLD = 16 * K / EPT;                  // COL: active loader threads
  constexpr int NP = (K + 63) / 64;                  // ROW: passes
  uint32_t rc[AXIS == CAFEQ_AXIS_COL ? EPT / 4 : NP];
  float4 rx[AXIS == CAFEQ_AXIS_COL ? EPT / 4 : NP];
  float4 rs[AXIS == CAFEQ_AXIS_COL ? EPT / 4 : NP];  // COL: .x only, one scale per chunk
  constexpr int TPR = K / EPT;                       // COL: threads per slab row; chunk j starts at column 4 (l % TPR) + 4 TPR j
  bool rok[AXIS == CAFEQ_AXIS_COL ? 1 : NP];

  auto issue = [&](int64_t t) {
    if (AXIS == CAFEQ_AXIS_COL) {
      const int tt = tid / TPR, c0 = (tid % TPR) * 4;
      const int64_t i = t + tt;
      rok[0] = tid < NLD && i < t1;
      if (rok[0]) {
#pragma unroll
        for (int j = 0; j < EPT / 4; ++j) {
          const int64_t col = f0 + c0 + 4 * TPR * j;
          rs[j].x = a.scales[i * (C / a.G) + col / a.G];
          rc[j] = *reinterpret_cast<const uint32_t*>(a.codes + i * C + col);
          rx[j] = *reinterpret_cast<const float4*>(a.X + i * C + col);
        }
      }
    } else {
#pragma unroll
      for (int pz = 0; pz < NP; ++pz) {
        const int r = pz * 64 + tid / 4;
        const int64_t c = t + 4 * (tid % 4);
        rok[pz] = r < K && c < t1;                  // tlen and chunk are multiples of 4
        if (rok[pz]) {
          const int64_t row = f0 + r;
          rs[pz] = *reinterpret_cast<const float4*>(a.scales + (row / a.G) * C + c);
          rc[pz] = *reinterpret_cast<const uint32_t*>(a.codes + row * C + c);
          rx[pz] = *reinterpret_cast<const float4*>(a.X + row * C + c);
        }
      }
    }
  };
  auto commit = [&]() {
    if (AXIS == CAFEQ_AXIS_COL) {
      if (tid < NLD) {
        const int tt = tid / TPR, c0 = (tid % TPR) * 4;
#pragma unroll
        for (int j = 0; j < EPT / 4; ++j) {
          float4 q = make_float4(0.f, 0.f, 0.f, 0.f), e = q;
          if (rok[0]) {
            const uint32_t cw = rc[j];
            q.x = __fmul_rn(float(int8_t(cw)), rs[j].x);
            q.y = __fmul_rn(float(int8_t(cw >> 8)), rs[j].x);
            q.z = __fmul_rn(float(int8_t(cw >> 16)), rs[j].x);
            q.w = __fmul_rn(float(int8_t(cw >> 24)), rs[j].x);
            e = make_float4(q.x - rx[j].x, q.y - rx[j].y, q.z - rx[j].z, q.w - rx[j].w);
          }
          *reinterpret_cast<float4*>(qs + tt * LD + c0 + 4 * TPR * j) = q;
          *reinterpret_cast<float4*>(es + tt * LD + c0 + 4 * TPR * j) = e;
        }
      }
    } else {
#pragma unroll
      for (int pz = 0; pz < NP; ++pz) {
        const int r = pz * 64 + tid / 4, tq = 4 * (tid % 4);
        if (r < K) {
          float q[4] = {0.f, 0.f, 0.f, 0.f}, e[4] = {0.f, 0.f, 0.f, 0.f};
          if (rok[pz]) {
            const uint32_t cw = rc[pz];
            q[0] = __fmul_rn(float(int8_t(cw)), rs[pz].x);
            q[1] = __fmul_rn(float(int8_t(cw >> 8)), rs[pz].y);
            q[2] = __fmul_rn(float(int8_t(cw >> 16)), rs[pz].z);
            q[3] = __fmul_rn(float(int8_t(cw >> 24)), rs[pz].w);
            e[0] = q[0] - rx[pz].x; e[1] = q[1] - rx[pz].y; e[2] = q[2] - rx[pz].z; e[3] = q[3] - rx[pz].w;
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            qs[(tq + j) * LD + r] = q[j];
            es[(tq + j) * LD + r] = e[j];
          }
        }
      }
    }
  };

  issue(t0);
  for (int64_t t = t0; t < t1; t += 16) {
    commit();
    __syncthreads();
    if (t + 16 < t1) issue(t + 16);
    if (active) {
      const float* pa = qs + h * LD + jt1 * 32 + ln;
      const float* pe = es + h * LD + jt1 * 32 + ln;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xa = pa[2 * e * LD];
        const float ea = TRIPLE ? pe[2 * e * LD] : 0.f;
#pragma unroll
        for (int u = 0; u < NU; ++u) {
          const int off = (2 * e + h) * LD + (wave + 4 * u) * 32 + ln;
          accS[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa, qs[off], accS[u], 0, 0, 0);
          accR[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa, es[off], accR[u], 0, 0, 0);
          if (TRIPLE) accT[TRIPLE ? u : 0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ea, es[off], accT[TRIPLE ? u : 0], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // partial[b][z][0|1(|2)][row][col]
  float* out = a.partial + ((size_t(b) * gridDim.z + z) * (TRIPLE ? 3 : 2)) * size_t(K) * K;
  if (active)
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int col = (wave + 4 * u) * 32 + ln;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = jt1 * 32 + 8 * (v / 4) + 4 * h + (v % 4);
        out[size_t(row) * K + col] = accS[u][v];
        out[size_t(K) * K + size_t(row) * K + col] = accR[u][v];
        if (TRIPLE) out[2 * size_t(K) * K + size_t(row) * K + col] = accT[TRIPLE ? u : 0][v];
      }
    }
}

// The same pair of Gram matrices for heads of 128 and 256 on the 16-bit matrix pipe.  Every float32 value -- the
// dequantized code Xq = fl(q s) and the error E = fl(Xq - X), the numbers the kernel above multiplies -- is split
// exactly into three bfloat16 parts (8 + 8 + 8 significant bits) and a product keeps the six part products of
// weight >= 2^-24 (hh, hm, mh, hl, lh, mm), float32 accumulation: the accuracy of the float32 instruction at 6/16 of
// its time.  So that the split is not repeated per 32-row stripe, a workgroup of eight waves owns a whole 128 x 128
// quadrant of a head's outputs (grid y: quadrant; 1 or 4 per head): per step of 16 contraction indices its 512
// threads each take eight consecutive contraction indices of one free index -- waves 0-3 the quadrant's row side
// (Xq), waves 4-7 its column side (Xq and E) -- dequantize, split, and store one 16-byte matrix-instruction operand
// per part into LDS ([part][half of the step][free index][8 contraction indices], two buffers, one barrier per step); then wave w
// accumulates the tiles (row tile w / 2; column tiles 2 (w % 2), 2 (w % 2) + 1) of S and R: 24 matrix instructions
// from 15 operand reads.  Partials in the layout of the kernel above.
constexpr int kG16PlaneB = 128 * 32;                 // one part of one side: 2 halves x 128 free indices x 8 bfloat16
constexpr int kG16BufB = 9 * kG16PlaneB;             // row side Xq, column side Xq, column side E: 3 parts each
constexpr size_t kG16Lds = 2 * kG16BufB;

__device__ __forceinline__ void split3_bf16(const float (&x)[8], uintx4& ph, uintx4& pm, uintx4& pl) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float x0 = x[2 * i], x1 = x[2 * i + 1];
    const uint32_t h = pack_bf16(x0, x1);
    const float r0 = x0 - bf16_lo_f32(h), r1 = x1 - bf16_hi_f32(h);
    const uint32_t m = pack_bf16(r0, r1);
    ph[i] = h;
    pm[i] = m;
    pl[i] = pack_bf16(r0 - bf16_lo_f32(m), r1 - bf16_hi_f32(m));
  }
}

template <int AXIS, int K>
__global__ __launch_bounds__(512) void gram_pair16_kernel(const GramArgs a) {
  static_assert(K == 128 || K == 256, "quadrants of 128");
  constexpr int QUADS = K / 128;
  extern __shared__ __align__(16) unsigned char gsm[];
  const int b = blockIdx.x, qI = blockIdx.y / QUADS, qJ = blockIdx.y % QUADS;
  const int z = blockIdx.z;                      // (row-block within head, chunk)
  const int qi = z / a.nchunk, ch = z % a.nchunk;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, h = lane >> 5;
  const int64_t t0 = int64_t(ch) * a.chunk;
  const int64_t t1 = t0 + a.chunk < a.tlen ? t0 + a.chunk : a.tlen;
  const int64_t f0 = AXIS == CAFEQ_AXIS_COL ? int64_t(b) * K : (int64_t(b) * a.rep + qi) * K;
  const int64_t C = a.cols;

  // loader role: side (uniform over a wave), free index, half of the step's 16 contraction indices
  // (sixteen neighbouring lanes share a half and take consecutive free indices: their 16-byte LDS stores form one
  // contiguous 256-byte run, like the operand reads)
  // Along columns a wave takes 64 consecutive columns of one half; along rows it takes both halves of 32 rows, so
  // that the two 32-byte pieces of a row's 64 bytes are asked for by one instruction.
  const int side = __builtin_amdgcn_readfirstlane(tid >> 8);
  const int idx = AXIS == CAFEQ_AXIS_COL ? (tid & 127) : ((tid >> 6) & 3) * 32 + ((lane >> 5) << 4) + (lane & 15);
  const int half = AXIS == CAFEQ_AXIS_COL ? ((tid >> 7) & 1) : ((lane >> 4) & 1);
  const int64_t fbase = f0 + 128 * (side ? qJ : qI);     // uniform over the wave
  const int64_t fidx = fbase + idx;
  struct LoadSet {
    float lx[8], lsc[8];
    uint32_t lc[AXIS == CAFEQ_AXIS_COL ? 8 : 2];
    bool lok[AXIS == CAFEQ_AXIS_COL ? 8 : 2];
  };
  auto issue = [&](LoadSet& L, int64_t t) {
    const int64_t tt = t + 8 * half;
    if (AXIS == CAFEQ_AXIS_COL) {
      // uniform bases of the step's first row plus 32-bit lane offsets (rows past the chunk: its last row, dropped)
      const int64_t tb = t < t1 ? t : t1 - 1;            // (a step past the chunk: its last row, all dropped)
      const float* bx = a.X + tb * C + fbase;
      const int8_t* bc = a.codes + tb * C + fbase;
      const float* bs = a.scales + tb * (C / a.G);
      const int gcol = int(fidx / a.G), cg = int(C / a.G);
      const int rmax = t < t1 ? int(t1 - 1 - t < 15 ? t1 - 1 - t : 15) : -1;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r0 = 8 * half + e;
        L.lok[e] = r0 <= rmax;
        const int r = r0 <= rmax ? r0 : (rmax >= 0 ? rmax : 0);
        const uint32_t off = uint32_t(r) * uint32_t(C) + uint32_t(idx);
        L.lc[e] = uint32_t(uint8_t(bc[off]));
        L.lx[e] = bx[off];
        L.lsc[e] = bs[uint32_t(r) * uint32_t(cg) + uint32_t(gcol)];
      }
    } else {
      const int64_t grow = fidx / a.G;
#pragma unroll
      for (int q4 = 0; q4 < 2; ++q4) {
        const int64_t c = tt + 4 * q4;
        L.lok[q4] = c < t1;                               // tlen and chunk are multiples of 4
        const int64_t cc = L.lok[q4] ? c : t1 - 4;
        L.lc[q4] = *reinterpret_cast<const uint32_t*>(a.codes + fidx * C + cc);
        const float4 vx = *reinterpret_cast<const float4*>(a.X + fidx * C + cc);
        const float4 vs = *reinterpret_cast<const float4*>(a.scales + grow * C + cc);
        L.lx[4 * q4] = vx.x; L.lx[4 * q4 + 1] = vx.y; L.lx[4 * q4 + 2] = vx.z; L.lx[4 * q4 + 3] = vx.w;
        L.lsc[4 * q4] = vs.x; L.lsc[4 * q4 + 1] = vs.y; L.lsc[4 * q4 + 2] = vs.z; L.lsc[4 * q4 + 3] = vs.w;
      }
    }
  };
  auto commit = [&](const LoadSet& L, unsigned char* buf) {
    float q[8], er[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      bool ok;
      int code;
      if (AXIS == CAFEQ_AXIS_COL) { ok = L.lok[e]; code = int(int8_t(L.lc[e])); }
      else { ok = L.lok[e >> 2]; code = int(int8_t(L.lc[e >> 2] >> (8 * (e & 3)))); }
      const float v = __fmul_rn(float(code), L.lsc[e]);
      q[e] = ok ? v : 0.f;
      er[e] = ok ? v - L.lx[e] : 0.f;
    }
    uintx4 ph, pm, pl;
    split3_bf16(q, ph, pm, pl);
    unsigned char* dst = buf + (side ? 3 * kG16PlaneB : 0) + half * (kG16PlaneB / 2) + idx * 16;
    *reinterpret_cast<uintx4*>(dst) = ph;
    *reinterpret_cast<uintx4*>(dst + kG16PlaneB) = pm;
    *reinterpret_cast<uintx4*>(dst + 2 * kG16PlaneB) = pl;
    if (side) {
      split3_bf16(er, ph, pm, pl);
      *reinterpret_cast<uintx4*>(dst + 3 * kG16PlaneB) = ph;
      *reinterpret_cast<uintx4*>(dst + 4 * kG16PlaneB) = pm;
      *reinterpret_cast<uintx4*>(dst + 5 * kG16PlaneB) = pl;
    }
  };

  const int ta = wave >> 1, tc0 = 2 * (wave & 1);
  floatx16 accS[2], accR[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int v = 0; v < 16; ++v) { accS[u][v] = 0.f; accR[u][v] = 0.f; }

  auto products = [&](const unsigned char* buf) {
    const unsigned char* pa = buf + h * (kG16PlaneB / 2) + (ta * 32 + ln) * 16;
    bf16x8 ax[3];
#pragma unroll
    for (int p = 0; p < 3; ++p) ax[p] = as_bf16x8(*reinterpret_cast<const uintx4*>(pa + p * kG16PlaneB));
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const unsigned char* pb = buf + 3 * kG16PlaneB + h * (kG16PlaneB / 2) + ((tc0 + u) * 32 + ln) * 16;
      bf16x8 bq[3], be[3];
#pragma unroll
      for (int p = 0; p < 3; ++p) {
        bq[p] = as_bf16x8(*reinterpret_cast<const uintx4*>(pb + p * kG16PlaneB));
        be[p] = as_bf16x8(*reinterpret_cast<const uintx4*>(pb + (3 + p) * kG16PlaneB));
      }
      // (smallest terms first)
      accS[u] = CAFEQ_MFMA_BF16(ax[1], bq[1], accS[u]);
      accS[u] = CAFEQ_MFMA_BF16(ax[0], bq[2], accS[u]);
      accS[u] = CAFEQ_MFMA_BF16(ax[2], bq[0], accS[u]);
      accS[u] = CAFEQ_MFMA_BF16(ax[0], bq[1], accS[u]);
      accS[u] = CAFEQ_MFMA_BF16(ax[1], bq[0], accS[u]);
      accS[u] = CAFEQ_MFMA_BF16(ax[0], bq[0], accS[u]);
      accR[u] = CAFEQ_MFMA_BF16(ax[1], be[1], accR[u]);
      accR[u] = CAFEQ_MFMA_BF16(ax[0], be[2], accR[u]);
      accR[u] = CAFEQ_MFMA_BF16(ax[2], be[0], accR[u]);
      accR[u] = CAFEQ_MFMA_BF16(ax[0], be[1], accR[u]);
      accR[u] = CAFEQ_MFMA_BF16(ax[1], be[0], accR[u]);
      accR[u] = CAFEQ_MFMA_BF16(ax[0], be[0], accR[u]);
    }
  };
  // Two steps of requests in flight (one register set per LDS buffer), and between two barriers a wave both
  // multiplies the step in one buffer and prepares the next step in the other (one barrier per step).  Requests
  // past the end of the chunk read in-range addresses and are dropped.
  LoadSet L0, L1;
  unsigned char* buf0 = gsm;
  unsigned char* buf1 = gsm + kG16BufB;
  issue(L0, t0);
  issue(L1, t0 + 16);
  commit(L0, buf0);
  for (int64_t t = t0; t < t1; t += 32) {
    __syncthreads();                       // buf0 holds step t; buf1's readers (step t - 16) are done
    issue(L0, t + 32);
    products(buf0);
    if (t + 16 < t1) {
      commit(L1, buf1);
      __syncthreads();                     // buf1 holds step t + 16; buf0's readers are done
      issue(L1, t + 48);
      products(buf1);
      if (t + 32 < t1) commit(L0, buf0);
    }
  }

  // partial[b][z][0|1][row][col]
  float* out = a.partial + ((size_t(b) * gridDim.z + z) * 2) * size_t(K) * K;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int col = 128 * qJ + (tc0 + u) * 32 + ln;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 128 * qI + ta * 32 + 8 * (v / 4) + 4 * h + (v % 4);
      out[size_t(row) * K + col] = accS[u][v];
      out[size_t(K) * K + size_t(row) * K + col] = accR[u][v];
    }
  }
}

// ---- paired quantization error from the Gram triples -------------------------------------------
// sums[(g)][m][K][K] (float64) = sum over the nchunk chunk partials of group g, m < 3
__global__ __launch_bounds__(256) void sum_triple_kernel(const float* __restrict__ partial, int nchunk, int K,
                                                          double* __restrict__ sums) {
  const int g = blockIdx.x, m = blockIdx.y;
  const size_t kk = size_t(K) * K;
  for (size_t e = size_t(blockIdx.z) * 256 + threadIdx.x; e < kk; e += size_t(gridDim.z) * 256) {
    double acc = 0.0;
    for (int c = 0; c < nchunk; ++c) acc += double(partial[((size_t(g) * nchunk + c) * 3 + m) * kk + e]);
    sums[(size_t(g) * 3 + m) * kk + e] = acc;
  }
}

// One workgroup per row-block q of V (head b = q / rep).  With SU = Uq^T Uq, RU = Uq^T E_U, TU = E_U^T E_U
// of head b and SV = Vq Vq^T, RV = Vq E_V^T, TV = E_V E_V^T of row-block q (E = dequantized - original):
//   Uq Vq - U V = Uq E_V + E_U V, so
//   ||Uq Vq - U V||_F^2 = tr(SU TV) + 2 tr(RU (RV - TV)) + tr(TU (SV - RV - RV^T + TV)),
//   ||U V||_F^2         = tr((SU - RU - RU^T + TU)(SV - RV - RV^T + TV));
// every term of the first line is at the scale of the rounding error (no cancellation).
__global__ __launch_bounds__(256) void pqe_trace_kernel(const double* __restrict__ su, const double* __restrict__ sv,
                                                         int K, int rep, double* __restrict__ perq) {
  __shared__ double red[2][4];
  const int q = blockIdx.x, b = q / rep;
  const size_t kk = size_t(K) * K;
  const double *SU = su + size_t(b) * 3 * kk, *RU = SU + kk, *TU = RU + kk;
  const double *SV = sv + size_t(q) * 3 * kk, *RV = SV + kk, *TV = RV + kk;
  double num = 0.0, den = 0.0;
  for (int e = threadIdx.x; e < K * K; e += 256) {
    const int i = e / K, j = e % K;
    const size_t ij = size_t(i) * K + j, ji = size_t(j) * K + i;
    const double vvt = SV[ji] - RV[ji] - RV[ij] + TV[ji];          // (V V^T)[j][i]
    const double utu = SU[ij] - RU[ij] - RU[ji] + TU[ij];          // (U^T U)[i][j]
    num += SU[ij] * TV[ji] + 2.0 * RU[ij] * (RV[ji] - TV[ji]) + TU[ij] * vvt;
    den += utu * vvt;
  }
  for (int m = 1; m < 64; m <<= 1) { num += __shfl_xor(num, m); den += __shfl_xor(den, m); }
  if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = num; red[1][threadIdx.x >> 6] = den; }
  __syncthreads();
  if (threadIdx.x == 0) {
    perq[2 * q] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    perq[2 * q + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

__global__ void pqe_finish_kernel(const double* __restrict__ perq, int nq, float* __restrict__ out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double num = 0.0, den = 0.0;
  for (int q = 0; q < nq; ++q) { num += perq[2 * q]; den += perq[2 * q + 1]; }
  out[0] = float(num);
  out[1] = float(den);
}

// Arguments of the Gauss-Jordan inversion kernel (one workgroup per block).
struct GjArgs {
  int mode, K, nz;
  const float* T;        // matrix to invert when partial == nullptr
  const float* partial;  // else [nb][nz][2][K][K]: chunk partials whose first matrix is summed and inverted
  const double* sum64 = nullptr;  // optional with partial: that float64 sum, already formed, [nb][K][K]
  const float* sum32 = nullptr;   // optional with sum64: the same sum rounded to float32 (gj_spd256_kernel reads this)
  double* work;          // unused by the register-resident kernel
  float* out;            // [nb][K][K]
  float* rho_row; float* rho_col;  // optional squared row / column norms of the inverse
  int* status; int status_stride, status_offset;
  const int* need;       // optional [nb][need_n]: blocks whose entries are all 0 are already done (see
  int need_n = 1;        // rotation_inverse_kernel, rotation_slice_kernel)
};

// Compile-time loop: f(integral_constant<int, I>) for I in [B, E).
template <int B, int E>
struct StaticFor {
  template <typename F>
  static __device__ __forceinline__ void run(F& f) {
    f(std::integral_constant<int, B>{});
    StaticFor<B + 1, E>::run(f);
  }
};
template <int E>
struct StaticFor<E, E> {
  template <typename F>
  static __device__ __forceinline__ void run(F&) {}
};

__device__ __forceinline__ uint32_t dpp_u32_max(uint32_t v, uint32_t o) { return v > o ? v : o; }
// maximum over the wave, returned as a wave-uniform value: DPP inside each row of 16 lanes,
// then the four row results are read back as scalars
__device__ __forceinline__ uint32_t wave_allmax_u32(uint32_t v) {
  v = dpp_u32_max(v, uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0xB1, 0xF, 0xF, true)));    // quad_perm [1,0,3,2]
  v = dpp_u32_max(v, uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x4E, 0xF, 0xF, true)));    // quad_perm [2,3,0,1]
  v = dpp_u32_max(v, uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x141, 0xF, 0xF, true)));   // row_half_mirror
  v = dpp_u32_max(v, uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x140, 0xF, 0xF, true)));   // row_mirror
  const uint32_t a = uint32_t(__builtin_amdgcn_readlane(int(v), 0)), b = uint32_t(__builtin_amdgcn_readlane(int(v), 16));
  const uint32_t c = uint32_t(__builtin_amdgcn_readlane(int(v), 32)), d = uint32_t(__builtin_amdgcn_readlane(int(v), 48));
  return dpp_u32_max(dpp_u32_max(a, b), dpp_u32_max(c, d));
}
// value held by lane `src` (wave-uniform) of a per-lane variable
__device__ __forceinline__ double read_lane(double x, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(x), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ float read_lane(float x, int src) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src));
}

// |x| as an unsigned key that orders like |x|: the leading 32 bits of the number without its sign
__device__ __forceinline__ uint32_t mag_bits(double x) { return uint32_t(__double2hiint(x)) & 0x7FFFFFFFu; }
__device__ __forceinline__ uint32_t mag_bits(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

__device__ __forceinline__ double fma_s(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float fma_s(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

// Register-resident in-place Gauss-Jordan inversion with partial pivoting, one workgroup per block.
// Thread (rt, ct) of an NRT x NCT thread grid keeps the RT x CT elements (rt + i*NRT, ct + j*NCT)
// in registers (both strides interleaved, so the LDS reads are either broadcasts or run over
// consecutive addresses).  No physical row swaps: the pivot of column k is the largest entry among
// the rows not yet used (PIV; for symmetric positive definite input, PIV == false, it is the diagonal
// entry), and the pivot order is a permutation undone on output.  One elimination
// step replaces column k by the unit vector e_p and adds multiples of row p / pivot to every row;
// row p itself goes through the same update with the multiplier (1 - pivot), which loses accuracy
// only for |pivot| >> 1, so the block is first scaled by a power of two to max |a_ij| in (1/2, 1].
// The steps of NB = 8 columns (a panel) are taken by the first wave on the K x NB panel alone -- rows
// in registers (lane l holds rows l, l + 64, ...), pivot search by DPP, pivot row through scalar lane
// reads, no barriers -- and their combined effect on the other columns, the rank-NB update
// R += C . X  (C: the panel after its steps minus the unit vectors of the pivot rows, X: the NB pivot
// rows as they were before the panel), is applied by all threads at once: three barriers per panel.
// A singular block keeps running (on infinities) and is zeroed at the end.
//   A = T_b (float32) when partial == nullptr, else the float64 sum over nz chunk partials
//   of S (first of the two K x K matrices of each partial).  out = A^-1 (zeros if singular).
template <int K, int RT, int CT, typename S, bool PIV>
__global__ __launch_bounds__((K / RT) * (K / CT)) void gj_panel_kernel(const GjArgs a) {
  constexpr int NRT = K / RT, NCT = K / CT, NTHR = NRT * NCT, NWAVE = (NTHR + 63) / 64;
  constexpr int NB = 8, NPH = NCT / NB, NRW = (K + 63) / 64;
  static_assert(NCT % NB == 0, "panel width");
  __shared__ __align__(16) S pan[2][K][NB];
  __shared__ __align__(16) S xrow[2][NB][K];
  __shared__ int pk[K], kinv[K];
  __shared__ int pvt[2][NB];
  __shared__ int deadflag;
  __shared__ S wred[16];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  if (a.need) {                           // uniform over the workgroup
    int any = 0;
    for (int i = 0; i < a.need_n; ++i) any |= a.need[b * a.need_n + i];
    if (!any) return;
  }
  const int rt = tid / NCT, ct = tid % NCT;
  S reg[RT][CT];
  if (a.partial == nullptr) {
    const float* src = a.T + size_t(b) * K * K;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
      for (int j = 0; j < CT; ++j) reg[i][j] = S(src[(rt + i * NRT) * K + ct + j * NCT]);
  } else if (a.sum64) {
    // one workgroup reading nz partials of its block is a long serial prologue when the blocks are few:
    // the float64 sum then comes from a kernel that spreads that work over the chip
    const double* src = a.sum64 + size_t(b) * K * K;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
      for (int j = 0; j < CT; ++j) reg[i][j] = S(src[(rt + i * NRT) * K + ct + j * NCT]);
  } else {
    const float* src = a.partial + size_t(b) * a.nz * 2 * K * K;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
      for (int j = 0; j < CT; ++j) reg[i][j] = 0;
    for (int z = 0; z < a.nz; ++z) {
      // float64 accumulation; the float elimination (K = 256) rounds the sum once
      double t[RT][CT];
#pragma unroll
      for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j) t[i][j] = double(src[size_t(z) * 2 * K * K + (rt + i * NRT) * K + ct + j * NCT]);
#pragma unroll
      for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j) reg[i][j] = S(double(reg[i][j]) + t[i][j]);
    }
  }
  S anorm = 0;
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j) anorm = fmax(anorm, fabs(reg[i][j]));
  for (int m = 1; m < 64; m <<= 1) anorm = fmax(anorm, __shfl_xor(anorm, m));
  if (lane == 0) wred[tid >> 6] = anorm;
  if (tid == 0) deadflag = 0;
  __syncthreads();
  anorm = 0;
  for (int i = 0; i < NWAVE; ++i) anorm = fmax(anorm, wred[i]);
  int ex = 0;
  (void)frexp(double(anorm), &ex);
  const S scale = S(ldexp(1.0, -ex));    // exact power of two; 1 if the block is all zero
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j) reg[i][j] *= scale;
  const S tol = anorm * scale * S(a.partial ? 1e-5 : (sizeof(S) == 8 ? 1e-12 : 1e-6));
  uint32_t usedbits = 0;   // first wave only: bit q = row lane + 64 q has been a pivot

  auto panels = [&](auto jj_c) {
    constexpr int jj = decltype(jj_c)::value;
    for (int h = 0; h < NPH; ++h) {
      const int buf = (jj * NPH + h) & 1;
      const int q_own = ct - h * NB;
      const bool owner = q_own >= 0 && q_own < NB;
      if (owner) {
#pragma unroll
        for (int i = 0; i < RT; ++i) pan[buf][rt + i * NRT][q_own] = reg[i][jj];
      }
      __syncthreads();
      if (tid < 64) {
        S prow[NRW][NB];
#pragma unroll
        for (int q = 0; q < NRW; ++q) {
          const int rr = lane + 64 * q;
#pragma unroll
          for (int c = 0; c < NB; ++c) prow[q][c] = rr < K ? pan[buf][rr < K ? rr : 0][c] : S(0);
        }
        int pivs[NB];
        bool dd = false;
#pragma unroll
        for (int s = 0; s < NB; ++s) {
          // pivot = (approximately) largest |entry| of the column among the unused rows: a 32-bit key
          // (leading bits of the magnitude, low byte 255 - row: ties go to the lowest row) reduced by DPP
          // (PIV == false, for symmetric positive definite input: the diagonal entry, no search)
          S colv[NRW];
          uint32_t key = 0x100u;
#pragma unroll
          for (int q = 0; q < NRW; ++q) colv[q] = prow[q][s];
          int p = jj * NCT + h * NB + s;
          if (PIV) {
            key = 0;
#pragma unroll
            for (int q = 0; q < NRW; ++q) {
              const int rr = lane + 64 * q;
              const uint32_t kk_ = (rr >= K || ((usedbits >> q) & 1u)) ? 0u
                                                                       : ((mag_bits(colv[q]) & 0xFFFFFF00u) | uint32_t(255 - rr));
              key = key > kk_ ? key : kk_;
            }
            key = wave_allmax_u32(key);
            p = (255 - int(key & 0xFFu)) & (K - 1);
          }
          const int pl = p & 63, pq = p >> 6;
          S pv = read_lane(colv[0], pl);
#pragma unroll
          for (int q = 1; q < NRW; ++q) {
            const S alt = read_lane(colv[q], pl);
            pv = pq == q ? alt : pv;
          }
          dd = dd || (key >> 8) == 0 || !((PIV ? S(fabs(pv)) : pv) > tol);
          // reciprocal of the pivot: hardware estimate (2^-22) + Newton steps to full precision
          S ipiv = S(__builtin_amdgcn_rcpf(float(pv)));
          ipiv = ipiv * (S(2) - pv * ipiv);
          if (sizeof(S) == 8) ipiv = ipiv * (S(2) - pv * ipiv);
          // row p of the panel, with the in-place 1 in the column of this step
          S rowp[NB];
#pragma unroll
          for (int c = 0; c < NB; ++c) {
            S mine = prow[0][c];
#pragma unroll
            for (int q = 1; q < NRW; ++q) mine = pq == q ? prow[q][c] : mine;
            rowp[c] = c == s ? S(1) : read_lane(mine, pl);
          }
#pragma unroll
          for (int q = 0; q < NRW; ++q) {
            const bool isp = (lane + 64 * q) == p;
            const S f = (isp ? S(1) - pv : -colv[q]) * ipiv;
#pragma unroll
            for (int c = 0; c < NB; ++c)
              prow[q][c] = c == s ? (isp ? S(1) : S(0)) + f : fma_s(f, rowp[c], prow[q][c]);
            usedbits |= uint32_t(isp) << q;
          }
          pivs[s] = p;
        }
        // hand over C = (panel after its steps) - (unit vectors of the pivot rows), and the pivots
#pragma unroll
        for (int q = 0; q < NRW; ++q) {
          const int rr = lane + 64 * q;
          if (rr < K) {
#pragma unroll
            for (int c = 0; c < NB; ++c) pan[buf][rr][c] = prow[q][c] - (rr == pivs[c] ? S(1) : S(0));
          }
        }
        if (lane == 0) {
#pragma unroll
          for (int c = 0; c < NB; ++c) {
            pvt[buf][c] = pivs[c];
            pk[jj * NCT + h * NB + c] = pivs[c];
          }
          if (dd) deadflag = 1;
        }
      }
      __syncthreads();
      // the owners of the pivot rows publish them as they were before the panel
#pragma unroll
      for (int c = 0; c < NB; ++c) {
        const int p = pvt[buf][c];
        const int prt = p % NRT;
        if constexpr (!PIV && NRT % NCT == 0) {
          // diagonal pivots p = jj NCT + h NB + c: the register row p / NRT does not depend on h and c
          constexpr int pi = (jj * NCT) / NRT;
          if (rt == prt) {
#pragma unroll
            for (int j = 0; j < CT; ++j) xrow[buf][c][ct + j * NCT] = reg[pi][j];
          }
        } else {
          // (one flat condition per register row: nesting the row test inside the thread test made the
          // compiler index the registers dynamically, through scratch memory)
          const int pi = p / NRT;
#pragma unroll
          for (int i = 0; i < RT; ++i)
            if (rt == prt && i == pi) {
#pragma unroll
              for (int j = 0; j < CT; ++j) xrow[buf][c][ct + j * NCT] = reg[i][j];
            }
        }
      }
      __syncthreads();
#pragma unroll 2
      for (int c = 0; c < NB; ++c) {
        S xv[CT], cr[RT];
#pragma unroll
        for (int j = 0; j < CT; ++j) xv[j] = xrow[buf][c][ct + j * NCT];
#pragma unroll
        for (int i = 0; i < RT; ++i) cr[i] = pan[buf][rt + i * NRT][c];
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
          for (int j = 0; j < CT; ++j) reg[i][j] = fma_s(cr[i], xv[j], reg[i][j]);
      }
      // a panel column becomes the panel's own result
      if (owner) {
        const int pq = pvt[buf][q_own];
#pragma unroll
        for (int i = 0; i < RT; ++i) {
          const int r = rt + i * NRT;
          reg[i][jj] = pan[buf][r][q_own] + (r == pq ? S(1) : S(0));
        }
      }
    }
  };
  StaticFor<0, CT>::run(panels);
  __syncthreads();
  const bool dead = deadflag != 0;
  if (a.status && tid == 0) a.status[size_t(b) * a.status_stride + a.status_offset] = dead ? 1 : 0;
  float* O = a.out + size_t(b) * K * K;
  if (dead) {
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
      for (int j = 0; j < CT; ++j) O[(rt + i * NRT) * K + ct + j * NCT] = 0.f;
    if (tid < K) {
      if (a.rho_row) a.rho_row[size_t(b) * K + tid] = 0.f;
      if (a.rho_col) a.rho_col[size_t(b) * K + tid] = 0.f;
    }
    return;
  }
  if (tid < K) kinv[pk[tid]] = tid;
  __syncthreads();
  // register (r, c) is element (kinv[r], pk[c]) of the inverse of the scaled block
  int ocol[CT];
#pragma unroll
  for (int j = 0; j < CT; ++j) ocol[j] = pk[ct + j * NCT];
#pragma unroll
  for (int i = 0; i < RT; ++i) {
    const int orow = kinv[rt + i * NRT];
    S rr = 0;
#pragma unroll
    for (int j = 0; j < CT; ++j) {
      reg[i][j] *= scale;
      O[orow * K + ocol[j]] = float(reg[i][j]);
      rr += reg[i][j] * reg[i][j];
    }
    if (a.rho_row) {
      for (int m = 1; m < NCT; m <<= 1) rr += __shfl_xor(rr, m);
      if (ct == 0) a.rho_row[size_t(b) * K + orow] = float(rr);
    }
  }
  if (a.rho_col) {
    // column norms from the block just written, one thread per column, rows in order (fixed summation order:
    // the result is reproducible run to run)
    __syncthreads();
    if (tid < K) {
      double c2 = 0;
      for (int i = 0; i < K; ++i) {
        const float v = O[i * K + tid];
        c2 += double(v) * v;
      }
      a.rho_col[size_t(b) * K + tid] = float(c2);
    }
  }
}

// The same inversion for a symmetric positive definite block of 256 in float32 (the Gram matrices of the adaptive
// rounding: diagonal pivots in natural order, so no permutation), as a block elimination in panels of 16 columns
// with everything but the 16 x 16 pivot block on the 16-bit matrix pipe.  With P the pivot block of panel t (rows
// and columns 16 t .. 16 t + 15 of the current matrix), D = P^-1, A the panel's other rows and X the sixteen pivot
// rows before the panel, sixteen elimination steps amount to
//     pivot block <- D,   panel (other rows) <- C = -A D,   pivot rows <- D X,   elsewhere  R <- R + C X,
// that is R += C' X on every row with C' = C (other rows) and D - I (pivot rows), and panel columns = C' + I.
// Only D needs the serial chain of steps (wave 0, one row per lane, pivot row through scalar lane reads; 16 lanes
// busy); C and the update are products of operands split exactly into three bfloat16 parts, the six part products
// of weight >= 2^-24 kept (as in gram_pair16_kernel).  Wave w of eight keeps rows 32 w .. 32 w + 31 as eight
// accumulator tiles: lane (ln, h) holds column 32 j + ln of tile j and rows 32 w + 8 (r / 4) + 4 h + r % 4,
// r = 0..15.  While wave 0 inverts P, the wave that holds the pivot rows (wave t / 2) splits them into the B
// operands of the update.  The contraction index c of the update is spread over the two lane halves as the
// accumulator layout delivers it -- half h takes c = 4 h + i and 8 + 4 h + i, i = 0..3 -- so that C^T = (-D^T) A^T
// comes out of the matrix pipe already in A-operand form (row 32 w + ln in lane ln), and the pivot rows' eight
// values per lane and tile are one 16-byte B operand; C in accumulator form, for the panel's own columns, is the
// same product with the operands exchanged.
__global__ __launch_bounds__(512) void gj_spd256_kernel(const GjArgs a) {
  constexpr int K = 256, NB = 16;
  __shared__ __align__(16) float pan[2][K][NB];
  constexpr int kXbB = 3 * 2 * K * 16;   // B operands of one panel's pivot rows: [part][lane half][column][8 rows]
  __shared__ __align__(16) unsigned char xb[2 * kXbB];
  __shared__ float dsm[2][16][17];       // D, float32
  __shared__ int deadflag, ready;        // ready: panels handed over so far
  __shared__ float wred[8];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6, ln = lane & 31, h = lane >> 5;
  if (a.need) {                           // uniform over the workgroup
    int any = 0;
    for (int i = 0; i < a.need_n; ++i) any |= a.need[b * a.need_n + i];
    if (!any) return;
  }
  const int rbase = 32 * w + 4 * h;       // row of register r: rbase + 8 (r / 4) + r % 4
  floatx16 reg[8];
  if (a.partial == nullptr || a.sum32) {
    // (float32 input: all 128 requests of a lane land in their registers, none waits for a conversion)
    const float* src = (a.partial == nullptr ? a.T : a.sum32) + size_t(b) * K * K;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) reg[j][r] = src[(rbase + 8 * (r >> 2) + (r & 3)) * K + 32 * j + ln];
  } else if (a.sum64) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        reg[j][r] = float(a.sum64[size_t(b) * K * K + size_t(rbase + 8 * (r >> 2) + (r & 3)) * K + 32 * j + ln]);
  } else {
    const float* src = a.partial + size_t(b) * a.nz * 2 * K * K;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        double acc = 0;
        for (int z = 0; z < a.nz; ++z)
          acc += double(src[size_t(z) * 2 * K * K + size_t(rbase + 8 * (r >> 2) + (r & 3)) * K + 32 * j + ln]);
        reg[j][r] = float(acc);
      }
  }
  float anorm = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) anorm = fmaxf(anorm, fabsf(reg[j][r]));
  for (int m = 1; m < 64; m <<= 1) anorm = fmaxf(anorm, __shfl_xor(anorm, m));
  if (lane == 0) wred[w] = anorm;
  if (tid == 0) deadflag = 0;
  __syncthreads();
  anorm = 0;
  for (int i = 0; i < 8; ++i) anorm = fmaxf(anorm, wred[i]);
  int ex = 0;
  (void)frexp(double(anorm), &ex);
  const float scale = float(ldexp(1.0, -ex));    // exact power of two; 1 if the block is all zero
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) reg[j][r] *= scale;
  const float tol = anorm * scale * (a.partial ? 1e-5f : 1e-6f);

  // (every panel is a compile-time variant: tile and register indices are constants)
  // the panel's columns, as they are now, into pan[half] (lanes that hold them: ln - 16 half in 0..15)
  auto own_write = [&](auto t_c) __attribute__((always_inline)) {
    constexpr int half = decltype(t_c)::value % 2, jt = decltype(t_c)::value / 2;
    const int q_own = ln - NB * half;
    if (q_own >= 0 && q_own < NB) {
#pragma unroll
      for (int r = 0; r < 16; ++r) pan[half][rbase + 8 * (r >> 2) + (r & 3)][q_own] = reg[jt][r];
    }
  };
  // wave 0: D = P^-1 in place, P = rows 16 t .. of pan[buf]; row (lane % 16) of the pivot block per lane (the
  // upper lanes repeat the lower sixteen)
  auto chain = [&](const int t, const int buf) __attribute__((always_inline)) {
    float prow[NB];
#pragma unroll
    for (int c4 = 0; c4 < NB / 4; ++c4) {
      const float4 v = *reinterpret_cast<const float4*>(&pan[buf][NB * t + (lane & 15)][4 * c4]);
      prow[4 * c4] = v.x; prow[4 * c4 + 1] = v.y; prow[4 * c4 + 2] = v.z; prow[4 * c4 + 3] = v.w;
    }
    bool dd = false;
#pragma unroll
    for (int s = 0; s < NB; ++s) {
      const float pv = read_lane(prow[s], s);
      dd = dd || !(pv > tol);
      // reciprocal of the pivot: hardware estimate (2^-22) + one Newton step
      float ipiv = __builtin_amdgcn_rcpf(pv);
      ipiv = ipiv * (2.f - pv * ipiv);
      float rowp[NB];
#pragma unroll
      for (int c = 0; c < NB; ++c) rowp[c] = c == s ? 1.f : read_lane(prow[c], s);
      const bool isp = (lane & 15) == s;
      const float f = (isp ? 1.f - pv : -prow[s]) * ipiv;
#pragma unroll
      for (int c = 0; c < NB; ++c)
        prow[c] = c == s ? (isp ? 1.f : 0.f) + f : fma_s(f, rowp[c], prow[c]);
    }
    if (lane < 16) {
#pragma unroll
      for (int c = 0; c < NB; ++c) dsm[buf][lane][c] = prow[c];
    }
    if (dd && lane == 0) deadflag = 1;
  };
  // The wave that holds them splits the pivot rows 16 t + c, as they are now, into the B operands xb[half].
  // Lane (ln, h) holds, for each of its columns, c = 8 g + 4 h + i (g = 0, 1; i = 0..3) in register
  // 4 (2 half + g) + i: the eight contraction indices of lane half h, in operand order.
  auto publish = [&](auto half_c) __attribute__((always_inline)) {
    constexpr int half = decltype(half_c)::value;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float xv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) xv[e] = reg[j][8 * half + e];
      uintx4 xh, xm, xl;
      split3_bf16(xv, xh, xm, xl);
      unsigned char* dst = xb + half * kXbB + (size_t(h) * K + 32 * j + ln) * 16;
      *reinterpret_cast<uintx4*>(dst) = xh;
      *reinterpret_cast<uintx4*>(dst + 2 * K * 16) = xm;
      *reinterpret_cast<uintx4*>(dst + 4 * K * 16) = xl;
    }
  };
  // Panel t = 2 jt + half, entered with pan[half], xb[half] and dsm[half] ready.  Every wave first updates the
  // tile that holds the next panel and hands that panel's columns over, so that wave 0 can invert the next pivot
  // block, after its own share of the update, while the slower waves are still multiplying: one barrier per panel.
  // (Measured without effect: a raised priority for wave 0; the inversion ahead of the rest of wave 0's update.)
  auto panel = [&](auto t_c) __attribute__((always_inline)) {
    constexpr int t = decltype(t_c)::value, half = t % 2, jt = t / 2, buf = half, nhalf = 1 - half, c0 = NB * half;
    constexpr int nt = t + 1, njt = nt / 2;
    constexpr bool has_next = nt < K / NB;
    const int q_own = ln - c0;
    const bool owner = q_own >= 0 && q_own < NB;
    float av[8], dv[8];
    const float4 a_lo = *reinterpret_cast<const float4*>(&pan[buf][32 * w + ln][8 * h]);
    const float4 a_hi = *reinterpret_cast<const float4*>(&pan[buf][32 * w + ln][8 * h + 4]);
    av[0] = a_lo.x; av[1] = a_lo.y; av[2] = a_lo.z; av[3] = a_lo.w;
    av[4] = a_hi.x; av[5] = a_hi.y; av[6] = a_hi.z; av[7] = a_hi.w;
#pragma unroll
    for (int e = 0; e < 8; ++e) dv[e] = owner ? -dsm[buf][8 * h + e][owner ? q_own : 0] : 0.f;
    uintx4 uh, um, ul;
    split3_bf16(av, uh, um, ul);
    const bf16x8 p0 = as_bf16x8(uh), p1 = as_bf16x8(um), p2 = as_bf16x8(ul);
    split3_bf16(dv, uh, um, ul);
    const bf16x8 d0 = as_bf16x8(uh), d1 = as_bf16x8(um), d2 = as_bf16x8(ul);
    floatx16 ct, cn;
#pragma unroll
    for (int v = 0; v < 16; ++v) { ct[v] = 0.f; cn[v] = 0.f; }
    // C^T (rows of the panel's columns c0 + c, column = this wave's row ln): operand order (-D^T, A^T)
    ct = CAFEQ_MFMA_BF16(d1, p1, ct);
    ct = CAFEQ_MFMA_BF16(d0, p2, ct);
    ct = CAFEQ_MFMA_BF16(d2, p0, ct);
    ct = CAFEQ_MFMA_BF16(d0, p1, ct);
    ct = CAFEQ_MFMA_BF16(d1, p0, ct);
    ct = CAFEQ_MFMA_BF16(d0, p0, ct);
    // C in accumulator form, valid in the owner lanes: operand order (A, -D)
    cn = CAFEQ_MFMA_BF16(p1, d1, cn);
    cn = CAFEQ_MFMA_BF16(p0, d2, cn);
    cn = CAFEQ_MFMA_BF16(p2, d0, cn);
    cn = CAFEQ_MFMA_BF16(p0, d1, cn);
    cn = CAFEQ_MFMA_BF16(p1, d0, cn);
    cn = CAFEQ_MFMA_BF16(p0, d0, cn);
    float cv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cv[e] = ct[8 * half + e];
    if (w == jt && owner) {
      // this lane's row is pivot row q_own: D - I there
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int c = 8 * (e >> 2) + 4 * h + (e & 3);
        cv[e] = dsm[buf][q_own][c] - (c == q_own ? 1.f : 0.f);
      }
    }
    split3_bf16(cv, uh, um, ul);
    const bf16x8 a0 = as_bf16x8(uh), a1 = as_bf16x8(um), a2 = as_bf16x8(ul);
    auto update = [&](auto j_c) __attribute__((always_inline)) {
      constexpr int j = decltype(j_c)::value;
      const unsigned char* pb = xb + buf * kXbB + (size_t(h) * K + 32 * j + ln) * 16;
      const bf16x8 b0 = as_bf16x8(*reinterpret_cast<const uintx4*>(pb));
      const bf16x8 b1 = as_bf16x8(*reinterpret_cast<const uintx4*>(pb + 2 * K * 16));
      const bf16x8 b2 = as_bf16x8(*reinterpret_cast<const uintx4*>(pb + 4 * K * 16));
      // (smallest terms first)
      floatx16 d = reg[j];
      d = CAFEQ_MFMA_BF16(a1, b1, d);
      d = CAFEQ_MFMA_BF16(a0, b2, d);
      d = CAFEQ_MFMA_BF16(a2, b0, d);
      d = CAFEQ_MFMA_BF16(a0, b1, d);
      d = CAFEQ_MFMA_BF16(a1, b0, d);
      d = CAFEQ_MFMA_BF16(a0, b0, d);
      reg[j] = d;
    };
    auto others = [&](auto j_c) __attribute__((always_inline)) {
      if constexpr (!has_next || decltype(j_c)::value != njt) update(j_c);
    };
    if constexpr (has_next) {
      update(std::integral_constant<int, njt>{});
      // (the next panel's columns lie in the other half of the lanes of tile njt: the replacement of this
      // panel's own columns below does not touch them)
      own_write(std::integral_constant<int, nt>{});
      // (every lane of the wave stores the count: each lane's own panel entries are released by its own store)
      if (w == njt) __hip_atomic_store(&ready, nt, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    StaticFor<0, 8>::run(others);
    // a panel column becomes the panel's own result: C' + I (D in the pivot rows)
    if (owner) {
#pragma unroll
      for (int r = 0; r < 16; ++r) cn[r] += (rbase + 8 * (r >> 2) + (r & 3)) == NB * t + q_own ? 1.f : 0.f;
      if (w == jt) {
#pragma unroll
        for (int e = 0; e < 8; ++e) cn[8 * half + e] = dsm[buf][8 * (e >> 2) + 4 * h + (e & 3)][q_own];
      }
      reg[jt] = cn;
    }
    if constexpr (has_next) {
      if (w == njt) publish(std::integral_constant<int, nhalf>{});
      if (w == 0) {
        // the pivot block of the next panel is part of what wave njt handed over; the wait is bounded (a wave
        // that never saw the hand-over marks the block as failed and goes on)
        int spins = 0;
        while (__hip_atomic_load(&ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < nt && spins < (1 << 22)) {
          __builtin_amdgcn_s_sleep(1);
          ++spins;
        }
        if (spins >= (1 << 22) && lane == 0) deadflag = 1;
        chain(nt, nhalf);
      }
    }
    __syncthreads();
  };
  own_write(std::integral_constant<int, 0>{});
  if (tid == 0) ready = 0;
  __syncthreads();
  if (w == 0) {
    chain(0, 0);
    publish(std::integral_constant<int, 0>{});
  }
  __syncthreads();
  StaticFor<0, K / NB>::run(panel);
  __syncthreads();
  const bool dead = deadflag != 0;
  if (a.status && tid == 0) a.status[size_t(b) * a.status_stride + a.status_offset] = dead ? 1 : 0;
  float* O = a.out + size_t(b) * K * K;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = rbase + 8 * (r >> 2) + (r & 3);
    float rr = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float v = dead ? 0.f : reg[j][r] * scale;
      O[size_t(row) * K + 32 * j + ln] = v;
      rr += v * v;
    }
    if (a.rho_row) {
      for (int m = 1; m < 32; m <<= 1) rr += __shfl_xor(rr, m);
      if (ln == 0) a.rho_row[size_t(b) * K + row] = rr;
    }
  }
  if (a.rho_col) {
    // column norms from the block just written, one thread per column, rows in order
    __syncthreads();
    if (tid < K) {
      double c2 = 0;
      for (int i = 0; i < K; ++i) {
        const float v = O[i * K + tid];
        c2 += double(v) * v;
      }
      a.rho_col[size_t(b) * K + tid] = float(c2);
    }
  }
}

// R_b = float64 sum over the chunk partials of the second matrix of each partial; C_b = I.
__global__ __launch_bounds__(256) void sum_r_init_c_kernel(const float* __restrict__ partial, int nz, int K,
                                                            float* __restrict__ R, float* __restrict__ C) {
  const int b = blockIdx.x;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < K * K; e += gridDim.y * 256) {
    const float* p = partial + size_t(b) * nz * 2 * K * K + size_t(K) * K + e;
    double acc = 0;
    for (int z = 0; z < nz; ++z) acc += double(p[size_t(z) * 2 * K * K]);
    R[size_t(b) * K * K + e] = float(acc);
    C[size_t(b) * K * K + e] = (e / K == e % K) ? 1.f : 0.f;
  }
}


// Float64-accumulating batched product for the iterative refinement of the K = 256 solve:
// C_b (double) = alpha * A_b B_b + beta * C_b, A and B float or double, on the float64 matrix instruction
// (v_mfma_f64_16x16x4_f64: the vector pipe's float64 rate at a sixth of the operand traffic; a version on vector
// multiply-adds, 2 x 4 results per thread, was bound by its LDS reads: 18 us against 12-15).  A 32 x 64 tile per
// workgroup (the few blocks of a k = 256 workload then give one workgroup per compute unit) of four
// waves, wave w the 16 x 16 tiles (w / 2, 2 (w % 2)) and (w / 2, 2 (w % 2) + 1); chunks of 64 contraction indices
// through LDS, the next chunk's requests in flight while one is multiplied; K a multiple of 64.  (All four chunks
// of K = 256 requested at the start measured the same.)  Operand layouts: lane l gives A[i = l % 16][k = l / 16] and B[k = l / 16][j = l % 16];
// its four results are rows l / 16 + 4 r (r = 0..3) of column l % 16.
typedef double doublex4 __attribute__((ext_vector_type(4)));
template <typename AT, typename BT>
__global__ __launch_bounds__(256) void bgemm_f64mfma_kernel(const AT* __restrict__ A, const BT* __restrict__ B,
                                                             double* __restrict__ C, int K, double alpha, double beta) {
  constexpr int LC = 64;
  __shared__ double sa[32][LC + 2];   // [i][l]   (row strides chosen so that the operand reads of 32 lanes cover
  __shared__ double sb[LC][80];       // [l][j]    all banks once)
  const int tpc = K / 64, tpr = K / 32;
  const int b = blockIdx.x / (tpr * tpc), tile = blockIdx.x % (tpr * tpc);
  const int i0 = (tile / tpc) * 32, j0 = (tile % tpc) * 64;
  const AT* Ab = A + size_t(b) * K * K;
  const BT* Bb = B + size_t(b) * K * K;
  double* Cb = C + size_t(b) * K * K;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, li = lane & 15, lk = lane >> 4;
  const int ti = w >> 1, tj0 = 2 * (w & 1);
  doublex4 acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[t][r] = 0.0;
  AT pa[8];
  BT pb[16];
  auto fetch = [&](int l0) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int e = tid + 256 * q;
      pa[q] = Ab[(i0 + e / LC) * K + l0 + e % LC];
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int e = tid + 256 * q;
      pb[q] = Bb[(l0 + e / 64) * K + j0 + e % 64];
    }
  };
  fetch(0);
  for (int l0 = 0; l0 < K; l0 += LC) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int e = tid + 256 * q;
      sa[e / LC][e % LC] = double(pa[q]);
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int e = tid + 256 * q;
      sb[e / 64][e % 64] = double(pb[q]);
    }
    __syncthreads();
    if (l0 + LC < K) fetch(l0 + LC);
#pragma unroll
    for (int s4 = 0; s4 < LC / 4; ++s4) {
      const double av = sa[16 * ti + li][4 * s4 + lk];
      const double b0 = sb[4 * s4 + lk][16 * tj0 + li];
      const double b1 = sb[4 * s4 + lk][16 * (tj0 + 1) + li];
      acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, b0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, b1, acc[1], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      double* dst = Cb + (i0 + 16 * ti + lk + 4 * r) * K + j0 + 16 * (tj0 + t) + li;
      *dst = alpha * acc[t][r] + (beta != 0.0 ? beta * *dst : 0.0);
    }
}

// S64, R64 and a second copy of R64 (the residual's starting value) from the chunk partials; optionally S64
// rounded to float32.
__global__ __launch_bounds__(256) void sum_partials64_kernel(const float* __restrict__ partial, int nz, int K,
                                                              double* __restrict__ S64, double* __restrict__ R64,
                                                              double* __restrict__ res, float* __restrict__ S32) {
  const int b = blockIdx.x;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < K * K; e += gridDim.y * 256) {
    const float* p = partial + size_t(b) * nz * 2 * K * K + e;
    double s = 0, r = 0;
    for (int z = 0; z < nz; ++z) {
      s += double(p[size_t(z) * 2 * K * K]);
      r += double(p[size_t(z) * 2 * K * K + size_t(K) * K]);
    }
    S64[size_t(b) * K * K + e] = s;
    if (S32) S32[size_t(b) * K * K + e] = float(s);
    R64[size_t(b) * K * K + e] = r;
    res[size_t(b) * K * K + e] = r;
  }
}
// ---- blocks of 256 near a (scaled) rotation: Newton-Schulz rounds on the matrix cores before any elimination.
// X0 = T^T / alpha with alpha = ||T_b||_F^2 / K is the exact inverse of a rotation scaled by any factor and a
// good start near one.  grid (nb, K / 32): workgroup (b, s) writes rows 32 s .. of X0 (columns of T).
__global__ __launch_bounds__(1024) void ns_init_kernel(const float* __restrict__ T, float* __restrict__ X0,
                                                       float* __restrict__ X0copy, int K) {
  __shared__ float tile[256 * 33];
  __shared__ double red[16];
  const int b = blockIdx.x, s0 = blockIdx.y * 32, tid = threadIdx.x;
  const float* Tb = T + size_t(b) * K * K;
  double acc = 0;
  for (int e = tid * 4; e < K * K; e += 1024 * 4) {
    const float4 v = *reinterpret_cast<const float4*>(Tb + e);
    acc += double(v.x) * v.x + double(v.y) * v.y + double(v.z) * v.z + double(v.w) * v.w;
  }
  for (int m = 1; m < 64; m <<= 1) acc += __shfl_xor(acc, m);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  // tile[j][ii] = T[j][s0 + ii]
  for (int e = tid; e < K * 32; e += 1024) {
    const int j = e >> 5, ii = e & 31;
    tile[j * 33 + ii] = Tb[size_t(j) * K + s0 + ii];
  }
  __syncthreads();
  double f2 = 0;
  for (int w = 0; w < 16; ++w) f2 += red[w];
  const float inv_alpha = f2 > 0 ? float(double(K) / f2) : 0.f;
  float* Xb = X0 + size_t(b) * K * K;
  float* Xc = X0copy + size_t(b) * K * K;      // (where the rounds' result lands: a block that needs none keeps X0)
  for (int e = tid; e < K * 32; e += 1024) {
    const int ii = e / K, j = e % K;
    const float x = tile[j * 33 + ii] * inv_alpha;
    Xb[size_t(s0 + ii) * K + j] = x;
    Xc[size_t(s0 + ii) * K + j] = x;
  }
}
// F = ||I - Y_b||_F per block, Y = T X.  mode 0 (after the first product): skip[b] = 1 when !(F <= thresh) -- such a
// block is hopeless for the rounds --, 2 when F <= done_thresh already (a rotation: the start is the inverse), else 0;
// the rounds leave blocks with skip != 0 alone.  mode 1 (after the last product): need[b] = skip[b] == 1 ||
// !(F <= thresh): the elimination takes those, the others are done (status 0).  Comparisons written so that a NaN
// fails them.  grid: nb.
__global__ __launch_bounds__(1024) void ns_flag_kernel(const float* __restrict__ Y, int K, int mode, float thresh,
                                                       float done_thresh, int* __restrict__ skip,
                                                       int* __restrict__ need, int* __restrict__ status) {
  __shared__ double red[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (mode == 1 && skip[b] == 1) {
    if (tid == 0) need[b] = 1;
    return;
  }
  const float* Yb = Y + size_t(b) * K * K;
  double acc = 0;
  for (int e = tid * 4; e < K * K; e += 1024 * 4) {
    const float4 v = *reinterpret_cast<const float4*>(Yb + e);
    const int r = e / K, c = e % K;
    const double d0 = double(v.x) - (r == c ? 1.0 : 0.0), d1 = double(v.y) - (r == c + 1 ? 1.0 : 0.0);
    const double d2 = double(v.z) - (r == c + 2 ? 1.0 : 0.0), d3 = double(v.w) - (r == c + 3 ? 1.0 : 0.0);
    acc += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
  }
  for (int m = 1; m < 64; m <<= 1) acc += __shfl_xor(acc, m);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    double f2 = 0;
  for (int w = 0; w < 16; ++w) f2 += red[w];
    const bool ok = f2 <= double(thresh) * double(thresh);
    if (mode == 0) {
      skip[b] = !ok ? 1 : (f2 <= double(done_thresh) * double(done_thresh) ? 2 : 0);
    } else {
      need[b] = ok ? 0 : 1;
      if (ok && status) status[b] = 0;
    }
  }
}
__global__ __launch_bounds__(256) void eye64_kernel(double* __restrict__ X, int K, int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  const int e = int(i % (int64_t(K) * K));
  X[i] = (e / K == e % K) ? 1.0 : 0.0;
}
__global__ __launch_bounds__(256) void add64_kernel(const double* __restrict__ D, int64_t n, float* __restrict__ X) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) X[i] = float(double(X[i]) + D[i]);
}
__global__ __launch_bounds__(256) void eye_minus_kernel(const double* __restrict__ X, int K, int64_t n,
                                                         float* __restrict__ C) {
  const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  const int e = int(i % (int64_t(K) * K));
  C[i] = float(((e / K == e % K) ? 1.0 : 0.0) - X[i]);
}

}  // namespace

namespace {
// Fast path of the blockwise inverse for blocks that are rotations to float32 accuracy -- the paper's
// initialisation of the transform: the inverse is then the transpose.  One workgroup per block, one wave
// per 32 x 32 tile: T goes to LDS in both orientations (row stride K + 1 words: rows and columns are both
// read without bank conflicts), R = I - T T^T is formed on the float32 matrix pipe, and if max |R| is at the
// level of its own accumulation noise (2e-6) the block is finished here: Tinv = T^T, its squared row /
// column norms, status 0, need[b] = 0.  Any other block is left to the elimination kernel (need[b] = 1),
// which skips the finished ones.  (Newton rounds X <- X + X R on this pipe were tried for blocks a little
// further from a rotation: each round leaves about 3e-6 of relative error, the noise of R; not kept.)
template <int K>
__global__ __launch_bounds__((K / 32) * (K / 32) * 64) void rotation_inverse_kernel(
    const float* __restrict__ T, float* __restrict__ Tinv, float* __restrict__ rho_row, float* __restrict__ rho_col,
    int* __restrict__ status, int* __restrict__ need) {
  constexpr int NTL = K / 32, NW = NTL * NTL, NTHR = NW * 64, LD = K + 1;
  extern __shared__ __align__(16) float nsm[];
  float* bufT = nsm;                 // T[i][l]
  float* bufX = nsm + K * LD;        // T^T[l][j]
  float* red = bufX + K * LD;        // [NW]
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5, wi = wave / NTL, wj = wave % NTL;
  const float* Tb = T + size_t(b) * K * K;
  for (int e = tid * 4; e < K * K; e += NTHR * 4) {
    const float4 v = *reinterpret_cast<const float4*>(Tb + e);
    const int r = e / K, c = e % K;
    float* d = bufT + r * LD + c;
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    bufX[(c + 0) * LD + r] = v.x; bufX[(c + 1) * LD + r] = v.y;
    bufX[(c + 2) * LD + r] = v.z; bufX[(c + 3) * LD + r] = v.w;
  }
  __syncthreads();
  // cheap necessary condition first: rows of unit length (most blocks that are no rotations leave here)
  {
    float dev = 0.f;
    if (tid < K) {
      float n2 = 0.f;
      for (int c = 0; c < K; ++c) { const float x = bufX[c * LD + tid]; n2 = fmaf(x, x, n2); }
      dev = fabsf(n2 - 1.f);
      if (!(dev <= 3.0e38f)) dev = INFINITY;
    }
    dev = cluster_allmax<64>(dev);
    if (lane == 0) red[wave] = dev;
    __syncthreads();
    float dmax = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) dmax = fmaxf(dmax, red[w]);
    __syncthreads();
    if (!(dmax <= 4e-6f)) {
      if (tid == 0) need[b] = 1;
      return;
    }
  }
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  {
    const float* pa = bufT + (wi * 32 + ln) * LD + h;   // a(l, i) = T[i][l], l = 2 s + h
    const float* pb = bufX + h * LD + wj * 32 + ln;      // b(l, j) = T^T[l][j]
#pragma unroll 8
    for (int s2 = 0; s2 < K / 2; ++s2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * s2], pb[2 * s2 * LD], acc, 0, 0, 0);
  }
  float m = 0.f;
  bool bad = false;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = wi * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = wj * 32 + ln;
    const float ar = fabsf((i == j ? 1.f : 0.f) - acc[v]);
    bad = bad || !(ar <= 3.0e38f);             // infinity or not a number
    m = fmaxf(m, ar);
  }
  if (bad) m = INFINITY;
  m = cluster_allmax<64>(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  float rmax = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) rmax = fmaxf(rmax, red[w]);
  const bool ok = rmax <= 2e-6f;
  if (tid == 0) need[b] = ok ? 0 : 1;
  if (!ok) return;
  float* O = Tinv + size_t(b) * K * K;
  for (int e = tid; e < K * K; e += NTHR) O[e] = bufX[(e / K) * LD + (e % K)];
  if (tid < K) {
    float rr = 0.f, rc = 0.f;
    for (int c = 0; c < K; ++c) {
      const float x = bufX[tid * LD + c], d = bufX[c * LD + tid];
      rr = fmaf(x, x, rr); rc = fmaf(d, d, rc);
    }
    if (rho_row) rho_row[size_t(b) * K + tid] = rr;
    if (rho_col) rho_col[size_t(b) * K + tid] = rc;
  }
  if (status && tid == 0) status[b] = 0;
}
// The same for blocks of 128 with four workgroups per block, one per slice of 32 rows of T (one workgroup per
// block keeps sixteen waves on one compute unit's float32 matrix pipe for 10 us; the 112 blocks of the 9B-shaped
// pair leave more than half of the chip idle).  Every slice loads the whole block (transposed, into LDS), checks
// its own rows -- unit length, then its 32 x 128 slice of R = I - T T^T, one 32 x 32 tile per wave -- and, if
// they pass, writes its share of the result: columns 32 s .. of Tinv = T^T, their squared norms, and the squared
// norms of the rows 32 s .. of Tinv.  need[4 b + s] = 0 / 1; a block with any slice failing is redone as a whole
// by the elimination kernel, which runs afterwards and overwrites what the passing slices wrote.
__global__ __launch_bounds__(256) void rotation_slice_kernel(const float* __restrict__ T, float* __restrict__ Tinv,
                                                             float* __restrict__ rho_row, float* __restrict__ rho_col,
                                                             int* __restrict__ status, int* __restrict__ need) {
  constexpr int K = 128, LD = K + 1;
  extern __shared__ __align__(16) float nsm[];
  float* bufX = nsm;                 // T^T[l][j]
  float* red = bufX + K * LD;        // [4]
  const int b = blockIdx.x >> 2, sl = blockIdx.x & 3;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, h = lane >> 5;
  const float* Tb = T + size_t(b) * K * K;
  for (int e = tid * 4; e < K * K; e += 256 * 4) {
    const float4 v = *reinterpret_cast<const float4*>(Tb + e);
    const int r = e / K, c = e % K;
    bufX[(c + 0) * LD + r] = v.x; bufX[(c + 1) * LD + r] = v.y;
    bufX[(c + 2) * LD + r] = v.z; bufX[(c + 3) * LD + r] = v.w;
  }
  __syncthreads();
  // squared lengths of this slice's rows of T (= columns of Tinv) and of its columns (= rows of Tinv): eight
  // threads per vector, sixteen terms each, combined through LDS in fixed order
  float* part = red + 4;             // [2][8][32]
  {
    const int i = sl * 32 + (tid & 31), q = tid >> 5;
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const float x = bufX[(16 * q + c) * LD + i];   // T[i][16 q + c]
      const float y = bufX[i * LD + 16 * q + c];     // T[16 q + c][i]
      a0 = fmaf(x, x, a0);
      a1 = fmaf(y, y, a1);
    }
    part[q * 32 + (tid & 31)] = a0;
    part[256 + q * 32 + (tid & 31)] = a1;
  }
  __syncthreads();
  float n2row = 0.f, n2col = 0.f;
  // cheap necessary condition first: rows of unit length
  {
    float dev = 0.f;
    if (tid < 32) {
#pragma unroll
      for (int q = 0; q < 8; ++q) { n2row += part[q * 32 + tid]; n2col += part[256 + q * 32 + tid]; }
      dev = fabsf(n2row - 1.f);
      if (!(dev <= 3.0e38f)) dev = INFINITY;
    }
    dev = cluster_allmax<64>(dev);
    if (lane == 0) red[wave] = dev;
    __syncthreads();
    const float dmax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    if (!(dmax <= 4e-6f)) {
      if (tid == 0) need[blockIdx.x] = 1;
      return;
    }
  }
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  {
    const float* pa = bufX + h * LD + sl * 32 + ln;      // a(l, i) = T[i][l] = T^T[l][i], l = 2 s + h
    const float* pb = bufX + h * LD + wave * 32 + ln;    // b(l, j) = T^T[l][j]
#pragma unroll 8
    for (int s2 = 0; s2 < K / 2; ++s2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * s2 * LD], pb[2 * s2 * LD], acc, 0, 0, 0);
  }
  float m = 0.f;
  bool bad = false;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = sl * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = wave * 32 + ln;
    const float ar = fabsf((i == j ? 1.f : 0.f) - acc[v]);
    bad = bad || !(ar <= 3.0e38f);
    m = fmaxf(m, ar);
  }
  if (bad) m = INFINITY;
  m = cluster_allmax<64>(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  const float rmax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const bool ok = rmax <= 2e-6f;
  if (tid == 0) need[blockIdx.x] = ok ? 0 : 1;
  if (!ok) return;
  // Tinv[j][i] = T[i][j] for the slice's i: 32 consecutive floats of every row j
  float* O = Tinv + size_t(b) * K * K + sl * 32;
  for (int e = tid; e < K * 32; e += 256) O[(e >> 5) * K + (e & 31)] = bufX[(e >> 5) * LD + sl * 32 + (e & 31)];
  if (tid < 32) {
    const int i = sl * 32 + tid;
    if (rho_col) rho_col[size_t(b) * K + i] = n2row;      // column i of Tinv is row i of T
    if (rho_row) rho_row[size_t(b) * K + i] = n2col;      // row i of Tinv is column i of T
  }
  if (status && tid == 0) status[b] = 0;
}
// Warm start for the learning loops, where the transform moves a little per iteration and the previous
// inverse X_0 is at hand: Newton's iteration  X <- X + X (I - T X), one workgroup per block, one wave per
// 32 x 32 tile, T and X in LDS; residuals on the float32 matrix pipe, corrections with bfloat16 operands.  The residual R = I - T X is measured every round;
// at the level of its own accumulation noise (4e-6) X stands, a round that promises max|R^2| <= 4e-6 (by
// K max|R|^2 or by the squared Frobenius norm) is the last, and a block whose residual is not a safe
// contraction (Frobenius norm >= 1/2) or is not done in three rounds is left to the elimination kernel
// (need[b] = 1).  The result carries the noise of R, about 3e-6 relative --
// below the 16-bit operand parts the loss pass makes of it, but above the elimination's float32 rounding, so
// the inverse a loop hands back to its caller is always recomputed by the elimination.
template <int K>
__global__ __launch_bounds__((K / 32) * (K / 32) * 64) void newton_inverse_kernel(const float* __restrict__ T,
                                                                                   float* __restrict__ X,
                                                                                   int* __restrict__ status,
                                                                                   int* __restrict__ need) {
  constexpr int NTL = K / 32, NW = NTL * NTL, NTHR = NW * 64, LD = K + 1;
  extern __shared__ __align__(16) float nsm[];
  float* bufT = nsm;                 // T[i][l], later R transposed in bfloat16 (rtb)
  uint16_t* rtb = reinterpret_cast<uint16_t*>(nsm);
  constexpr int LDB = K + 8;         // bfloat16 elements per row of rtb: 16-byte aligned rows
  float* bufX = nsm + K * LD;        // X[l][j]
  float* red = bufX + K * LD;        // [2 NW]: max |R| and sum R^2 of each wave's tile
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, h = lane >> 5, wi = wave / NTL, wj = wave % NTL;
  const float* Tb = T + size_t(b) * K * K;
  float* Xb = X + size_t(b) * K * K;
  auto load = [&](const float* src, float* dst) {
    for (int e = tid * 4; e < K * K; e += NTHR * 4) {
      const float4 v = *reinterpret_cast<const float4*>(src + e);
      float* d = dst + (e / K) * LD + (e % K);
      d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    }
  };
  load(Tb, bufT);
  load(Xb, bufX);
  __syncthreads();
  bool ok = false, changed = false;
#pragma unroll 1
  for (int it = 0; it < 3; ++it) {
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    {
      const float* pa = bufT + (wi * 32 + ln) * LD + h;   // a(l, i) = T[i][l], l = 2 s + h
      const float* pb = bufX + h * LD + wj * 32 + ln;      // b(l, j) = X[l][j]
#pragma unroll 8
      for (int s2 = 0; s2 < K / 2; ++s2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * s2], pb[2 * s2 * LD], acc, 0, 0, 0);
    }
    float r[16], m = 0.f, q = 0.f;
    bool bad = false;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = wi * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = wj * 32 + ln;
      r[v] = (i == j ? 1.f : 0.f) - acc[v];
      const float ar = fabsf(r[v]);
      bad = bad || !(ar <= 3.0e38f);           // infinity or not a number
      m = fmaxf(m, ar);
      q = fmaf(ar, ar, q);
    }
    if (bad) m = INFINITY;
    m = cluster_allmax<64>(m);
    q = wave_sum(q);
    if (lane == 0) { red[wave] = m; red[NW + wave] = q; }
    __syncthreads();                           // also: every wave has finished reading bufT
    float rmax = red[0], fro2 = red[NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) { rmax = fmaxf(rmax, red[w]); fro2 += red[NW + w]; }
    if (!(fro2 < 0.25f)) break;                // ||R||_2 <= ||R||_F; not a contraction to count on: elimination
    if (rmax <= 4e-6f) { ok = true; break; }   // the residual is float32 accumulation noise: X stands
    // The correction X R needs no more than 16-bit operands: what their rounding leaves (2^-8 of the
    // correction) is part of the next round's residual, and below float32 noise in the last round.
    // R goes to LDS transposed, in bfloat16, over the rows of the old T.
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int i0 = wi * 32 + 8 * g + 4 * h, j = wj * 32 + ln;
      uint2 pk;
      pk.x = pack_bf16(r[4 * g], r[4 * g + 1]);
      pk.y = pack_bf16(r[4 * g + 2], r[4 * g + 3]);
      *reinterpret_cast<uint2*>(rtb + j * LDB + i0) = pk;
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    {
      const float* pa = bufX + (wi * 32 + ln) * LD + 8 * h;          // a(l, i) = X[i][l], l = 16 s + 8 h + e
      const uint16_t* pb = rtb + (wj * 32 + ln) * LDB + 8 * h;       // b(l, j) = R[l][j] = RT[j][l]
#pragma unroll 4
      for (int s2 = 0; s2 < K / 16; ++s2) {
        const float* x = pa + 16 * s2;
        const bf16x8 av = as_bf16x8(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
        const bf16x8 bv = as_bf16x8(*reinterpret_cast<const uintx4*>(pb + 16 * s2));
        acc = CAFEQ_MFMA_BF16(av, bv, acc);
      }
    }
    float xn[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = wi * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = wj * 32 + ln;
      xn[v] = bufX[i * LD + j] + acc[v];
    }
    __syncthreads();                           // every wave has finished reading bufX and bufT
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = wi * 32 + 8 * (v / 4) + 4 * h + (v % 4), j = wj * 32 + ln;
      bufX[i * LD + j] = xn[v];
    }
    changed = true;
    if (fminf(float(K) * rmax * rmax, fro2) <= 4e-6f) { ok = true; break; }   // max |R^2| is below both
    load(Tb, bufT);                            // T again for the next round's residual
    __syncthreads();
  }
  __syncthreads();
  if (tid == 0) need[b] = ok ? 0 : 1;
  if (!ok) return;
  if (changed)
    for (int e = tid; e < K * K; e += NTHR) Xb[e] = bufX[(e / K) * LD + (e % K)];
  if (status && tid == 0) status[b] = 0;
}
}  // namespace

namespace {
int launch_gj(const GjArgs& a, int nb, hipStream_t st) {
  // the Gram matrices of the adaptive rounding are symmetric positive definite: no pivot search there
  const bool piv = a.partial == nullptr;
#define CAFEQ_GJ(K_, RT_, CT_, S_, THR_)                                                                      \
  if (piv) hipLaunchKernelGGL((gj_panel_kernel<K_, RT_, CT_, S_, true>), dim3(nb), dim3(THR_), 0, st, a);     \
  else hipLaunchKernelGGL((gj_panel_kernel<K_, RT_, CT_, S_, false>), dim3(nb), dim3(THR_), 0, st, a)
  switch (a.K) {
    case 32: CAFEQ_GJ(32, 4, 4, double, 64); break;
    case 64: CAFEQ_GJ(64, 4, 8, double, 128); break;
    case 128: CAFEQ_GJ(128, 4, 8, double, 512); break;
    case 256:
      if (piv) hipLaunchKernelGGL((gj_panel_kernel<256, 8, 16, float, true>), dim3(nb), dim3(512), 0, st, a);
      else hipLaunchKernelGGL(gj_spd256_kernel, dim3(nb), dim3(512), 0, st, a);
      break;
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
#undef CAFEQ_GJ
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
}  // namespace

int launch_gram(int axis, const float* X, const int8_t* codes, const float* scales, int64_t rows, int64_t cols,
                int K, int G, int nb, int rep, int64_t chunk, int nchunk, bool triple, float* partial, hipStream_t st);
int launch_gram_pair(int axis, const float* X, const int8_t* codes, const float* scales, int64_t rows,
                     int64_t cols, int K, int G, int nb, int rep, int64_t chunk, int nchunk, float* partial,
                     hipStream_t st) {
  return launch_gram(axis, X, codes, scales, rows, cols, K, G, nb, rep, chunk, nchunk, false, partial, st);
}
// Paired quantization error from Gram triples.  partialU / partialV: 3 k x k matrices per (head, chunk) /
// (row-block, chunk); sums: 3 * (nb + nb*rep) * k * k doubles + 2 * nb * rep doubles.
int launch_pqe(const float* U, const float* V, int64_t rowsA, int64_t colsA, int64_t rowsB, int64_t colsB, int K,
               int GA, int GB, int nb, int rep, const int8_t* codesU, const float* scalesU, const int8_t* codesV,
               const float* scalesV, int64_t chunkA, int nchunkA, int64_t chunkB, int nchunkB, float* partialU,
               float* partialV, double* sums, float* out, hipStream_t st) {
  int rc = launch_gram(CAFEQ_AXIS_COL, U, codesU, scalesU, rowsA, colsA, K, GA, nb, 1, chunkA, nchunkA, true, partialU, st);
  if (rc) return rc;
  rc = launch_gram(CAFEQ_AXIS_ROW, V, codesV, scalesV, rowsB, colsB, K, GB, nb, rep, chunkB, nchunkB, true, partialV, st);
  if (rc) return rc;
  const size_t kk = size_t(K) * K;
  double* su = sums;
  double* sv = sums + size_t(nb) * 3 * kk;
  double* perq = sv + size_t(nb) * rep * 3 * kk;
  hipLaunchKernelGGL(sum_triple_kernel, dim3(nb, 3, 16), dim3(256), 0, st, partialU, nchunkA, K, su);
  hipLaunchKernelGGL(sum_triple_kernel, dim3(nb * rep, 3, 16), dim3(256), 0, st, partialV, nchunkB, K, sv);
  hipLaunchKernelGGL(pqe_trace_kernel, dim3(nb * rep), dim3(256), 0, st, su, sv, K, rep, perq);
  hipLaunchKernelGGL(pqe_finish_kernel, dim3(1), dim3(64), 0, st, perq, nb * rep, out);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}
int launch_gram(int axis, const float* X, const int8_t* codes, const float* scales, int64_t rows, int64_t cols,
                int K, int G, int nb, int rep, int64_t chunk, int nchunk, bool triple, float* partial, hipStream_t st) {
  GramArgs a;
  a.X = X; a.codes = codes; a.scales = scales; a.rows = rows; a.cols = cols; a.K = K; a.G = G;
  a.rep = axis == CAFEQ_AXIS_COL ? 1 : rep;
  a.tlen = axis == CAFEQ_AXIS_COL ? rows : cols;
  a.chunk = chunk; a.nchunk = nchunk; a.partial = partial;
  if (!triple && (K == 128 || K == 256)) {
    // heads of 128 and 256: the 16-bit kernel, one workgroup per (head, quadrant of 128 x 128, chunk)
    const dim3 g16(nb, (K / 128) * (K / 128), a.rep * nchunk);
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
      bool ok = true;
#define CAFEQ_ATTR16(AX, KK)                                                                                    \
  ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(gram_pair16_kernel<AX, KK>),                    \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, int(kG16Lds)) == hipSuccess
      CAFEQ_ATTR16(CAFEQ_AXIS_COL, 128); CAFEQ_ATTR16(CAFEQ_AXIS_COL, 256);
      CAFEQ_ATTR16(CAFEQ_AXIS_ROW, 128); CAFEQ_ATTR16(CAFEQ_AXIS_ROW, 256);
#undef CAFEQ_ATTR16
      if (!ok) return CAFEQ_ERR_LAUNCH;
      attr_set = true;
    }
    if (axis == CAFEQ_AXIS_COL) {
      if (K == 128) hipLaunchKernelGGL((gram_pair16_kernel<CAFEQ_AXIS_COL, 128>), g16, dim3(512), kG16Lds, st, a);
      else hipLaunchKernelGGL((gram_pair16_kernel<CAFEQ_AXIS_COL, 256>), g16, dim3(512), kG16Lds, st, a);
    } else {
      if (K == 128) hipLaunchKernelGGL((gram_pair16_kernel<CAFEQ_AXIS_ROW, 128>), g16, dim3(512), kG16Lds, st, a);
      else hipLaunchKernelGGL((gram_pair16_kernel<CAFEQ_AXIS_ROW, 256>), g16, dim3(512), kG16Lds, st, a);
    }
    CAFEQ_CHECK_LAUNCH();
    return CAFEQ_OK;
  }
  dim3 grid(nb, K / 32, a.rep * nchunk);
#define CAFEQ_GRAM(KK)                                                                                          \
  case KK:                                                                                                      \
    if (axis == CAFEQ_AXIS_COL) {                                                                               \
      if (triple) hipLaunchKernelGGL((gram_pair_kernel<CAFEQ_AXIS_COL, KK, true>), grid, dim3(256), 0, st, a);  \
      else hipLaunchKernelGGL((gram_pair_kernel<CAFEQ_AXIS_COL, KK, false>), grid, dim3(256), 0, st, a);        \
    } else {                                                                                                    \
      if (triple) hipLaunchKernelGGL((gram_pair_kernel<CAFEQ_AXIS_ROW, KK, true>), grid, dim3(256), 0, st, a);  \
      else hipLaunchKernelGGL((gram_pair_kernel<CAFEQ_AXIS_ROW, KK, false>), grid, dim3(256), 0, st, a);        \
    }                                                                                                           \
    break;
  switch (K) {
    CAFEQ_GRAM(32) CAFEQ_GRAM(64) CAFEQ_GRAM(128) CAFEQ_GRAM(256)
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
#undef CAFEQ_GRAM
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

// C_b = I - S_b^-1 R_b with S, R the float64 sums of the chunk partials.  Sinv, R: [nb][K][K]
// float32 scratch; work: 4 * nb * K * K doubles.  A singular S_b yields C_b = I and status 1.
// K <= 128: S is inverted in float64.  K == 256: S is inverted in float32 and the solution
// X = S^-1 R gets one step of iterative refinement with float64 residuals.
int launch_gj_solve(int K, int nb, int nz, const float* partial, double* work, float* Sinv, float* R,
                    float* out, int* status, int status_stride, int status_offset, hipStream_t st) {
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = nz; a.T = nullptr; a.partial = partial; a.work = work; a.out = Sinv;
  a.need = nullptr;
  a.rho_row = a.rho_col = nullptr; a.status = status; a.status_stride = status_stride;
  a.status_offset = status_offset;
  const size_t mat = size_t(nb) * K * K;
  double *S64 = work, *R64 = work + mat, *res = work + 2 * mat, *X64 = work + 3 * mat;
  if (K == 256 || nb <= 64) {
    // few blocks (always so for K = 256 shapes): the sums over the chunk partials are formed by the whole chip
    // (K == 256 does not use the float32 scratch R otherwise: it holds the rounded sum the elimination reads)
    float* S32 = K == 256 ? R : nullptr;
    hipLaunchKernelGGL(sum_partials64_kernel, dim3(nb, 32), dim3(256), 0, st, partial, nz, K, S64, R64, res, S32);
    CAFEQ_CHECK_LAUNCH();
    a.sum64 = S64;
    a.sum32 = S32;
  }
  int rc = launch_gj(a, nb, st);
  if (rc) return rc;
  if (K < 256) {
    hipLaunchKernelGGL(sum_r_init_c_kernel, dim3(nb, 16), dim3(256), 0, st, partial, nz, K, R, out);
    CAFEQ_CHECK_LAUNCH();
    return launch_bgemm(false, false, Sinv, R, out, K, nb, -1.f, 1.f, st);
  }
  const unsigned grid = unsigned(nb) * (K / 32) * (K / 64);
  hipLaunchKernelGGL((bgemm_f64mfma_kernel<float, double>), dim3(grid), dim3(256), 0, st, Sinv, R64, X64, K, 1.0, 0.0);
  hipLaunchKernelGGL((bgemm_f64mfma_kernel<double, double>), dim3(grid), dim3(256), 0, st, S64, X64, res, K, -1.0, 1.0);
  hipLaunchKernelGGL((bgemm_f64mfma_kernel<float, double>), dim3(grid), dim3(256), 0, st, Sinv, res, X64, K, 1.0, 1.0);
  const int64_t n = int64_t(mat);
  hipLaunchKernelGGL(eye_minus_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, X64, K, n, out);
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int launch_inverse256(const float* T, int nb, double* work, float* Tinv, float* rho_row, float* rho_col, int* status,
                      bool warm, hipStream_t st);
int launch_block_inverse(const float* T, int K, int nb, double* work, float* Tinv, float* rho_row,
                         float* rho_col, int* status, hipStream_t st) {
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = 0; a.T = T; a.partial = nullptr; a.work = work; a.out = Tinv;
  a.rho_row = rho_row; a.rho_col = rho_col; a.status = status; a.status_stride = 1; a.status_offset = 0;
  a.need = nullptr;
  if (K == 64 || K == 128) {
    // rotations (to float32 accuracy) are inverted by transposition; the elimination then only runs for
    // the blocks that are none (flags at the start of the work buffer)
    int* need = reinterpret_cast<int*>(work);
    const size_t lds = size_t(2 * K * (K + 1) + (K / 32) * (K / 32)) * sizeof(float);
    if (K == 128) {
      // four workgroups per block, one per slice of 32 rows (flags need[4 b + slice])
      const size_t lds4 = size_t(K * (K + 1) + 4 + 512) * sizeof(float);
      static std::atomic<bool> attr_set{false};
      if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(rotation_slice_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(lds4)) != hipSuccess)
          return CAFEQ_ERR_LAUNCH;
        attr_set = true;
      }
      hipLaunchKernelGGL(rotation_slice_kernel, dim3(4 * nb), dim3(256), lds4, st, T, Tinv, rho_row, rho_col, status, need);
      a.need_n = 4;
    } else {
      hipLaunchKernelGGL(rotation_inverse_kernel<64>, dim3(nb), dim3(256), lds, st, T, Tinv, rho_row, rho_col, status, need);
    }
    CAFEQ_CHECK_LAUNCH();
    a.need = need;
  }
  if (K != 256) return launch_gj(a, nb, st);
  return launch_inverse256(T, nb, work, Tinv, rho_row, rho_col, status, false, st);
}

// Blocks of 256.  Newton-Schulz rounds X <- 2 X - X (T X) on the float32 matrix pipe (batched products over the
// whole chip) from X0 = T^T / alpha (cold) or from the inverse already in Tinv (warm: inside a learning loop),
// accepted per block when ||I - T X||_F <= 3e-4 afterwards -- an a-posteriori bound, so a start that was not
// good enough only costs the rounds; blocks that are hopeless after the first product (||I - T X0||_F > 1.2) skip
// them, and so do blocks whose start already meets the bound (rotations).  Every other block is eliminated in float32 (one compute unit each, 283 us).  Either way one Newton step
// with float64 residuals follows and brings the result to float32 rounding accuracy (it squares the residual).
// work: 2 nb K K doubles; the rounds' two float32 matrices and the flags share it with the refinement's buffers.
int launch_inverse256(const float* T, int nb, double* work, float* Tinv, float* rho_row, float* rho_col, int* status,
                      bool warm, hipStream_t st) {
  constexpr int K = 256;
  int rc;
  const size_t mat = size_t(nb) * K * K;
  float* Xs = reinterpret_cast<float*>(work);
  float* Y = Xs + mat;
  int* hop = reinterpret_cast<int*>(reinterpret_cast<unsigned char*>(work) + 2 * mat * sizeof(double) -
                                    ((size_t(2 * nb) * sizeof(int) + 255) / 256) * 256);
  int* need = hop + nb;
  auto product_tx = [&](const float* X) { return launch_bgemm(false, false, T, X, Y, K, nb, 1.f, 0.f, st); };
  auto round = [&](const float* X, float* Xn) {   // Xn = 2 X - X Y
    return launch_bgemm(false, false, X, Y, Xn, K, nb, -1.f, 2.f, st, nullptr, X, hop);
  };
  if (!warm) {
    hipLaunchKernelGGL(ns_init_kernel, dim3(nb, K / 32), dim3(1024), 0, st, T, Xs, Tinv, K);
    CAFEQ_CHECK_LAUNCH();
    if ((rc = product_tx(Xs))) return rc;
    hipLaunchKernelGGL(ns_flag_kernel, dim3(nb), dim3(1024), 0, st, Y, K, 0, 1.2f, 3e-4f, hop, need, status);
    if ((rc = round(Xs, Tinv))) return rc;
    if ((rc = product_tx(Tinv))) return rc;
    if ((rc = round(Tinv, Xs))) return rc;
    if ((rc = product_tx(Xs))) return rc;
    if ((rc = round(Xs, Tinv))) return rc;
  } else {
    if ((rc = product_tx(Tinv))) return rc;
    hipLaunchKernelGGL(ns_flag_kernel, dim3(nb), dim3(1024), 0, st, Y, K, 0, 1.2f, 3e-4f, hop, need, status);
    if ((rc = round(Tinv, Xs))) return rc;
    if ((rc = product_tx(Xs))) return rc;
    if ((rc = round(Xs, Tinv))) return rc;
  }
  if ((rc = product_tx(Tinv))) return rc;
  hipLaunchKernelGGL(ns_flag_kernel, dim3(nb), dim3(1024), 0, st, Y, K, 1, 3e-4f, 0.f, hop, need, status);
  CAFEQ_CHECK_LAUNCH();
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = 0; a.T = T; a.partial = nullptr; a.work = work; a.out = Tinv;
  a.rho_row = a.rho_col = nullptr; a.status = status; a.status_stride = 1; a.status_offset = 0;
  a.need = need; a.need_n = 1;
  if ((rc = launch_gj(a, nb, st))) return rc;
  // one Newton step X <- X + X (I - T X) with float64 residuals
  double *res = work, *X64 = work + mat;
  const unsigned grid = unsigned(nb) * (K / 32) * (K / 64);
  const int64_t n = int64_t(mat);
  hipLaunchKernelGGL(eye64_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, res, K, n);
  hipLaunchKernelGGL((bgemm_f64mfma_kernel<float, float>), dim3(grid), dim3(256), 0, st, T, Tinv, res, K, -1.0, 1.0);
  hipLaunchKernelGGL((bgemm_f64mfma_kernel<float, double>), dim3(grid), dim3(256), 0, st, Tinv, res, X64, K, 1.0, 0.0);
  hipLaunchKernelGGL(add64_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, st, X64, n, Tinv);
  CAFEQ_CHECK_LAUNCH();
  if (rho_row && (rc = launch_rho(Tinv, K, nb, 1, rho_row, st))) return rc;
  if (rho_col && (rc = launch_rho(Tinv, K, nb, 0, rho_col, st))) return rc;
  return CAFEQ_OK;
}

// The inverse inside a learning loop: Tinv holds the previous iteration's inverse on entry.
int launch_block_inverse_warm(const float* T, int K, int nb, double* work, float* Tinv, int* status, hipStream_t st) {
  if (K == 256) return launch_inverse256(T, nb, work, Tinv, nullptr, nullptr, status, true, st);
  if (K != 64 && K != 128) return launch_block_inverse(T, K, nb, work, Tinv, nullptr, nullptr, status, st);
  int* need = reinterpret_cast<int*>(work);
  const size_t lds = size_t(2 * K * (K + 1) + 2 * (K / 32) * (K / 32)) * sizeof(float);
  if (K == 128) {
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(newton_inverse_kernel<128>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
        return CAFEQ_ERR_LAUNCH;
      attr_set = true;
    }
    hipLaunchKernelGGL(newton_inverse_kernel<128>, dim3(nb), dim3(1024), lds, st, T, Tinv, status, need);
  } else {
    hipLaunchKernelGGL(newton_inverse_kernel<64>, dim3(nb), dim3(256), lds, st, T, Tinv, status, need);
  }
  CAFEQ_CHECK_LAUNCH();
  GjArgs a;
  a.mode = 0; a.K = K; a.nz = 0; a.T = T; a.partial = nullptr; a.work = work; a.out = Tinv;
  a.rho_row = a.rho_col = nullptr; a.status = status; a.status_stride = 1; a.status_offset = 0;
  a.need = need;
  return launch_gj(a, nb, st);
}

}  // namespace cafeq
