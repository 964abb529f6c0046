// extern "C" entry points: argument validation and dispatch.  See include/cafeq.h.
#include <utility>
#include <vector>

#include "xform_core.hpp"
#include "loss_reduce.hpp"

using namespace cafeq;
namespace cafeq {
// (defined further down, next to the timing table)
int launch_grad_owner_timed(const GradOwnerJob* jobs, int n, int loss_kind, float beta, float lse_t, const double* lse_ms,
                            hipStream_t st, const LossArgs* fold);
int launch_grad_v2_timed(const CoreParams& p, hipStream_t st);
int launch_grad_pass_timed(int K, int axis, const CoreParams& p, hipStream_t st);
}  // namespace cafeq

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_mat(const cafeq_mat* m) {
  if (!m || !m->data) return CAFEQ_ERR_INVALID_ARG;
  if (m->dtype != CAFEQ_F32 && m->dtype != CAFEQ_BF16) return CAFEQ_ERR_INVALID_ARG;
  if (m->rows <= 0 || m->cols <= 0 || m->ld < m->cols) return CAFEQ_ERR_BAD_SHAPE;
  if (m->cols % 4 != 0) return CAFEQ_ERR_BAD_SHAPE;
  const int64_t ldm = m->dtype == CAFEQ_F32 ? 4 : 8;
  if (m->ld % ldm != 0 || !aligned16(m->data)) return CAFEQ_ERR_BAD_ALIGN;
  return CAFEQ_OK;
}

// allow_minmax: the call has kernels for the min/max grid of Eq. (1)
int check_cfg(const cafeq_quant_cfg* c, bool need_axis, bool allow_minmax = false) {
  if (!c) return CAFEQ_ERR_INVALID_ARG;
  if (c->bits < 2 || c->bits > 8 || c->group < 0) return CAFEQ_ERR_INVALID_ARG;
  if (need_axis && c->axis != CAFEQ_AXIS_COL && c->axis != CAFEQ_AXIS_ROW) return CAFEQ_ERR_INVALID_ARG;
  if (c->mode == CAFEQ_Q_ASYM_MINMAX) return allow_minmax ? CAFEQ_OK : CAFEQ_ERR_UNSUPPORTED;
  if (c->mode != CAFEQ_Q_SYM_ABSMAX) return CAFEQ_ERR_INVALID_ARG;
  return CAFEQ_OK;
}


// ---------------------------------------------------------------------------------------
// planning of one fused-core launch and its scratch layout
// ---------------------------------------------------------------------------------------
struct CorePlan {
  int K, G, L, NBLK, NGRP, nseg, nwg;
  int64_t nlines, naxis, mt_per_seg, n_mt, nslot;
  size_t slot_grad_floats;   // per slot
};

bool supported_block(int k) { return k == 32 || k == 64 || k == 128 || k == 256; }

// How the quantization groups of one matrix lie over the fused core's segments.  Groups of 32, 64, 128 or
// 256 are a compile-time parameter of the core (a segment holds whole groups).  Any longer group -- a whole
// channel, the per-channel setting of the paper's experiments, included -- spans `gspan` segments of `Gk`
// elements; the core then runs with one group per segment and the group's absmax is assembled from the
// segments' records (CoreParams::gspan).
struct GroupPlan {
  int G;       // group length along the axis
  int Gk;      // the core's compile-time group
  int gspan;   // segments per group
};
int resolve_group(const cafeq_quant_cfg* cfg, int64_t naxis, int K, GroupPlan* gp) {
  const int64_t g = cfg->group == 0 ? naxis : cfg->group;
  if (g <= 0 || naxis % g != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (g > (int64_t(1) << 30)) return CAFEQ_ERR_UNSUPPORTED;
  gp->G = int(g);
  if (g == 32 || g == 64 || g == 128 || g == 256) { gp->Gk = int(g); gp->gspan = 1; return CAFEQ_OK; }
  int L = K > 128 ? K : 128;
  if (g % L != 0) L = K;
  if (g < L || g % L != 0) return CAFEQ_ERR_UNSUPPORTED;
  gp->Gk = L; gp->gspan = int(g / L);
  return CAFEQ_OK;
}

// grad: the launch will ask for the fused gradient.  Without it, segments of up to 128 run two
// workgroups per compute unit.
int make_plan(int K, int G, int64_t nlines, int64_t naxis, CorePlan* pl, bool grad = true) {
  if (!supported_block(K)) return CAFEQ_ERR_UNSUPPORTED;
  if (!(G == 32 || G == 64 || G == 128 || G == 256)) return CAFEQ_ERR_UNSUPPORTED;
  pl->K = K; pl->G = G; pl->L = K > G ? K : G;
  if (naxis % pl->L != 0) return CAFEQ_ERR_BAD_SHAPE;
  pl->NBLK = pl->L / K; pl->NGRP = pl->L / G;
  pl->nlines = nlines; pl->naxis = naxis;
  pl->nseg = int(naxis / pl->L);
  pl->mt_per_seg = (nlines + kMacroLines - 1) / kMacroLines;
  pl->n_mt = pl->mt_per_seg * pl->nseg;
  const int per_cu = (!grad && pl->L <= 128) ? 2 : 1;
  int64_t nwg = std::min<int64_t>(pl->n_mt, int64_t(device_cu_count()) * per_cu);
  if (nwg > 8) nwg -= nwg % 8;
  pl->nwg = int(nwg);
  pl->nslot = pl->nwg + pl->nseg;
  pl->slot_grad_floats = size_t(pl->NBLK) * K * K;
  return CAFEQ_OK;
}

// The gradient pass of the two-pass scheme walks the axis in chunks of 128 inputs, two workgroups per
// compute unit (one for blocks of 256).
int make_grad_plan(int K, int64_t nlines, int64_t naxis, CorePlan* pl) {
  if (!supported_block(K)) return CAFEQ_ERR_UNSUPPORTED;
  if (naxis % 128 != 0) return CAFEQ_ERR_UNSUPPORTED;
  pl->K = K; pl->G = 0; pl->L = 128; pl->NBLK = 0; pl->NGRP = 0;
  pl->nlines = nlines; pl->naxis = naxis;
  pl->nseg = int(naxis / 128);
  pl->mt_per_seg = (nlines + kMacroLines - 1) / kMacroLines;
  pl->n_mt = pl->mt_per_seg * pl->nseg;
  int64_t nwg = std::min<int64_t>(pl->n_mt, int64_t(device_cu_count()) * (K == 256 ? 1 : 2));
  if (nwg > 8) nwg -= nwg % 8;
  // A whole number of workgroups per chunk, where the longest range gets no longer by it: no range then
  // straddles two chunks (one partial per workgroup instead of up to two) and all ranges are equal.
  {
    const int64_t per = nwg / pl->nseg;
    if (per >= 1 && pl->mt_per_seg % per == 0 && pl->mt_per_seg / per <= (pl->n_mt + nwg - 1) / nwg &&
        (per * pl->nseg) % 8 == 0)
      nwg = per * pl->nseg;
  }
  pl->nwg = int(nwg);
  pl->nslot = pl->nwg + pl->nseg;
  pl->slot_grad_floats = grad_pass_part_floats(K);
  return CAFEQ_OK;
}

struct Carver {
  char* base; size_t off;
  explicit Carver(void* b) : base(static_cast<char*>(b)), off(0) {}
  template <typename T> T* take(size_t n) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off = align_up(off + n * sizeof(T), 256);
    return p;
  }
};

// Whether the loss pass for (K, G) runs its forward contraction on two-part half-precision operands: the
// gradient-free kernel variant over 128 x 128 blocks with one block per segment, for grids of up to 4 bits
// (two float16 parts carry 22 of float32's 24 bits; the error that leaves in z / scale grows with the number of
// levels, so finer grids keep the six-product bfloat16 forward).
bool core_forward_f16(int K, int G, int bits) { return K == 128 && G <= 128 && bits <= 4; }

// Plans of one matrix for a call with / without gradient: `first` is the pass that computes the losses,
// `gpass` the pass that writes the gradient partials (== first when the gradient is fused into it).
// The gradient runs as a second pass over the weights, from the loss pass's arg-max records, where the fused
// kernel has no gradient (blocks of 256, groups of 256 with blocks of 64 or more), where the two passes are
// faster (blocks of 128), and for groups that span several segments.
// asym: the min/max grid of Eq. (1); its kernel variants are gradient-free, so the gradient always takes the
// second pass.
struct PassPlans { CorePlan first, gpass; GroupPlan gp; bool two, fused, v2, asym; };
bool is_minmax(const cafeq_quant_cfg* cfg) { return cfg->mode == CAFEQ_Q_ASYM_MINMAX; }
// levels and the surrogate's constant for either grid (Sec. 4.1: 1 / (2^b - 1)^2 for Eq. (1); a quarter of the
// squared step of the symmetric grid)
QGrid grid_for(const cafeq_quant_cfg* cfg) {
  if (!is_minmax(cfg)) return make_grid(cfg->bits);
  QGrid g;
  g.qmax = float((1 << cfg->bits) - 1);
  g.qmin = 0.f;
  return g;
}
float beta_for(const cafeq_quant_cfg* cfg, const QGrid& g) {
  return is_minmax(cfg) ? 1.f / (g.qmax * g.qmax) : 1.f / (4.f * g.qmax * g.qmax);
}
// The loss pass over prepared weights (loss_v2.hip): one workgroup of eight waves per compute unit,
// macro-tiles of 256 lines.
bool v2_eligible(const cafeq_mat* W, int K, const GroupPlan& gp, const cafeq_quant_cfg* cfg) {
  return W->prepared != nullptr && K == 128 && gp.Gk <= 128 && gp.gspan == 1 && cfg->bits <= 4 && !is_minmax(cfg);
}
// share: the matrix gets 1 / share of the chip's compute units (2: the members of a pair that run in one launch)
void make_v2_plan(CorePlan* pl, int share = 1) {
  pl->mt_per_seg = (pl->nlines + 255) / 256;
  pl->n_mt = pl->mt_per_seg * pl->nseg;
  int64_t nwg = std::min<int64_t>(pl->n_mt, int64_t(device_cu_count()) / share);
  if (nwg > 8) nwg -= nwg % 8;
  pl->nwg = int(nwg);
  pl->nslot = pl->nwg + pl->nseg;
}
int plan_passes(int K, const GroupPlan& gp, int64_t nlines, int64_t naxis, bool grad, PassPlans* pp,
                bool v2 = false, bool asym = false, int v2_share = 1) {
  pp->gp = gp;
  pp->v2 = v2;
  pp->asym = asym;
  const size_t fl = core_lds_bytes(K, gp.Gk, true);
  const bool fused_ok = fl != 0 && fl <= 160 * 1024 && gp.gspan == 1 && !(K == 128 && gp.Gk <= 128) && !asym;
  pp->two = grad && !fused_ok;
  pp->fused = grad && fused_ok;
  int rc = make_plan(K, gp.Gk, nlines, naxis, &pp->first, pp->fused);
  if (rc) return rc;
  if (v2) make_v2_plan(&pp->first, v2_share);
  if (pp->two) return make_grad_plan(K, nlines, naxis, &pp->gpass);
  pp->gpass = pp->first;
  return CAFEQ_OK;
}

// scratch of one matrix's passes
struct MemberWs {
  float *rG, *rGreal, *slot_grad, *fs, *fsi;
  uint16_t *pfwd, *pinv;
  float2 *rec, *grec;
  float2 *rec_mm, *grec_mm;   // min/max grid with groups that span segments
};
void carve_member(Carver& c, const PassPlans& pp, int nb, bool grad, bool want_rG, MemberWs* w) {
  const CorePlan& pl = pp.first;
  const bool big = pp.gp.gspan > 1;
  w->fs = c.take<float>(nb);
  w->fsi = c.take<float>(nb);
  w->pfwd = c.take<uint16_t>(size_t(nb) * kFwdPlanes * pl.K * pl.K);
  w->pinv = c.take<uint16_t>(size_t(nb) * kInvPlanes * pl.K * pl.K);
  w->rG = c.take<float>(want_rG ? size_t(pl.naxis / pl.G) : 0);
  w->rGreal = big && want_rG ? c.take<float>(size_t(pl.naxis / pp.gp.G)) : w->rG;
  w->slot_grad = c.take<float>(grad ? size_t(pp.gpass.nslot) * pp.gpass.slot_grad_floats : 0);
  w->rec = c.take<float2>((pp.two || big) ? size_t(pl.naxis / pl.G) * size_t(pl.nlines) : 0);
  w->grec = big ? c.take<float2>(size_t(pl.naxis / pp.gp.G) * size_t(pl.nlines)) : w->rec;
  const bool mm = big && pp.asym;
  w->rec_mm = c.take<float2>(mm ? size_t(pl.naxis / pl.G) * size_t(pl.nlines) : 0);
  w->grec_mm = c.take<float2>(mm ? size_t(pl.naxis / pp.gp.G) * size_t(pl.nlines) : 0);
  if (!mm) w->rec_mm = w->grec_mm = nullptr;
}

struct SingleWs {
  double* lse_ms; float* member_ref; float *rho, *slot_hdr, *mmid, *x1; MemberWs m; size_t bytes;
};
SingleWs carve_single(void* ws, const PassPlans& pp, int nb, bool grad) {
  Carver c(ws);
  SingleWs w;
  const CorePlan& pl = pp.first;
  w.lse_ms = c.take<double>(2);
  w.member_ref = c.take<float>(4);
  w.rho = c.take<float>(size_t(nb) * pl.K);
  w.slot_hdr = c.take<float>(size_t(pl.nslot) * kHdrFloats);
  w.mmid = c.take<float>(grad ? size_t(nb) * pl.K * pl.K : 0);
  w.x1 = c.take<float>(grad ? size_t(nb) * pl.K * pl.K : 0);
  carve_member(c, pp, nb, grad, true, &w.m);
  w.bytes = c.off;
  return w;
}

struct DualWs {
  double* lse_ms; float* member_ref; float *hdrA, *hdrB, *gp, *x1; MemberWs a, b; size_t bytes;
};
DualWs carve_dual(void* ws, const PassPlans& qa, const PassPlans& qb, int nb, bool grad) {
  Carver c(ws);
  DualWs w;
  const int K = qa.first.K;
  w.lse_ms = c.take<double>(2);
  w.member_ref = c.take<float>(4);   // [0]: member A, [1]: member B
  w.hdrA = c.take<float>(size_t(qa.first.nslot + qb.first.nslot) * kHdrFloats);   // A then B, contiguous
  w.hdrB = w.hdrA ? w.hdrA + size_t(qa.first.nslot) * kHdrFloats : nullptr;
  w.gp = c.take<float>(grad ? size_t(nb) * K * K : 0);
  w.x1 = c.take<float>(grad ? size_t(nb) * K * K : 0);
  carve_member(c, qa, nb, grad, false, &w.a);
  carve_member(c, qb, nb, grad, false, &w.b);
  w.bytes = c.off;
  return w;
}

int check_xform(const cafeq_xform* x, bool need_inv) {
  if (!x || !x->T || (need_inv && !x->Tinv)) return CAFEQ_ERR_INVALID_ARG;
  if (!supported_block(x->k)) return CAFEQ_ERR_UNSUPPORTED;
  if (x->nb <= 0 || x->rep <= 0) return CAFEQ_ERR_BAD_SHAPE;
  if (!aligned16(x->T) || (x->Tinv && !aligned16(x->Tinv))) return CAFEQ_ERR_BAD_ALIGN;
  return CAFEQ_OK;
}

int check_axis_len(const cafeq_mat* W, const cafeq_xform* x, int axis) {
  if (axis == CAFEQ_AXIS_COL) {
    if (x->rep != 1 || W->cols != int64_t(x->nb) * x->k) return CAFEQ_ERR_BAD_SHAPE;
  } else if (axis == CAFEQ_AXIS_ROW) {
    if (W->rows != int64_t(x->nb) * x->rep * x->k) return CAFEQ_ERR_BAD_SHAPE;
  } else {
    return CAFEQ_ERR_INVALID_ARG;
  }
  return CAFEQ_OK;
}

// Transform blocks of 2, 4, 8 or 16: a run of 32 / k of them is one block-diagonal block of 32, which is how every
// entry point below runs them (embed into scratch, call itself with blocks of 32, gather the gradient's diagonal
// sub-blocks).  small_m: 32 / k for those sizes, 0 for any other.
int small_m(int k) { return (k == 2 || k == 4 || k == 8 || k == 16) ? 32 / k : 0; }
struct SmallWs { float *T32, *P32, *G32; int* st32; void* sub; size_t head; };
SmallWs carve_small(void* ws, int64_t nb32) {
  Carver c(ws);
  SmallWs w;
  w.T32 = c.take<float>(size_t(nb32) * 1024);
  w.P32 = c.take<float>(size_t(nb32) * 1024);
  w.G32 = c.take<float>(size_t(nb32) * 1024);
  w.st32 = c.take<int>(size_t(nb32));
  w.head = c.off;
  w.sub = ws ? static_cast<char*>(ws) + c.off : nullptr;
  return w;
}
// blocks of 32 that a small-block transform over `naxis` indices makes (0: not a whole number)
int64_t small_nb32(const cafeq_xform* x, int64_t naxis) {
  if (naxis % 32 != 0 || naxis != int64_t(x->nb) * x->rep * x->k) return 0;
  return naxis / 32;
}
int check_small_xform(const cafeq_xform* x, bool need_inv) {
  if (!x || !x->T || (need_inv && !x->Tinv)) return CAFEQ_ERR_INVALID_ARG;
  if (x->nb <= 0 || x->rep <= 0) return CAFEQ_ERR_BAD_SHAPE;
  if (!aligned16(x->T) || (x->Tinv && !aligned16(x->Tinv))) return CAFEQ_ERR_BAD_ALIGN;
  return CAFEQ_OK;
}
size_t orth_ws_any(int k, int nb) {
  if (!small_m(k)) return orth_workspace_bytes(k, nb);
  const int64_t nb32 = int64_t(nb) * k / 32;
  return carve_small(nullptr, nb32).head + orth_workspace_bytes(32, int(nb32));
}

struct AdaptivePlan {
  GroupPlan ga, gb;
  int nchunkA, nchunkB;
  int64_t chunkA, chunkB;
  CorePlan planU, planV;
  size_t partial_floats, rec_entries, grec_entries, bytes;
};
void split_contraction(int64_t tlen, int units, int64_t* chunk, int* nchunk) {
  // aim at about two workgroups per compute unit, chunks of at least 64 and a multiple of 16
  int64_t want = (2 * int64_t(device_cu_count()) + units - 1) / units;
  want = std::max<int64_t>(1, std::min<int64_t>(want, (tlen + 63) / 64));
  int64_t ch = (tlen + want - 1) / want;
  ch = (ch + 15) / 16 * 16;
  *chunk = ch;
  *nchunk = int((tlen + ch - 1) / ch);
}
struct AdaptiveWs {
  float* partial; double* work; float *Cmat, *Sinv, *Rsum; uint16_t* planes; float2 *rec, *grec;
};
AdaptiveWs carve_adaptive(void* ws, const AdaptivePlan& ap, int k, int nb, size_t* bytes) {
  Carver c(ws);
  AdaptiveWs w;
  w.partial = c.take<float>(ap.partial_floats);
  w.work = c.take<double>(size_t(nb) * k * 4 * k);
  w.Cmat = c.take<float>(size_t(nb) * k * k);
  w.Sinv = c.take<float>(size_t(nb) * k * k);
  w.Rsum = c.take<float>(size_t(nb) * k * k);
  w.planes = c.take<uint16_t>(size_t(nb) * kFwdPlanes * k * k);
  w.rec = c.take<float2>(ap.rec_entries);
  w.grec = c.take<float2>(ap.grec_entries);
  if (bytes) *bytes = c.off;
  return w;
}
int plan_adaptive(const cafeq_quant_cfg* cfg, int k, int nb, int rep, int64_t rowsA, int64_t colsA,
                  int64_t rowsB, int64_t colsB, AdaptivePlan* ap) {
  int rc;
  if (!supported_block(k)) return CAFEQ_ERR_UNSUPPORTED;
  if ((rc = resolve_group(cfg, colsA, k, &ap->ga))) return rc;
  if ((rc = resolve_group(cfg, rowsB, k, &ap->gb))) return rc;
  if ((rc = make_plan(k, ap->ga.Gk, rowsA, colsA, &ap->planU, false))) return rc;
  if ((rc = make_plan(k, ap->gb.Gk, colsB, rowsB, &ap->planV, false))) return rc;
  split_contraction(rowsA, nb * (k / 32), &ap->chunkA, &ap->nchunkA);
  split_contraction(colsB, nb * rep * (k / 32), &ap->chunkB, &ap->nchunkB);
  const size_t nz = size_t(std::max(ap->nchunkA, rep * ap->nchunkB));
  ap->partial_floats = size_t(nb) * nz * 2 * k * k;
  // groups that span several segments: records of the requantization's first sweep
  ap->rec_entries = std::max(ap->ga.gspan > 1 ? size_t(colsA / ap->ga.Gk) * size_t(rowsA) : 0,
                             ap->gb.gspan > 1 ? size_t(rowsB / ap->gb.Gk) * size_t(colsB) : 0);
  ap->grec_entries = std::max(ap->ga.gspan > 1 ? size_t(colsA / ap->ga.G) * size_t(rowsA) : 0,
                              ap->gb.gspan > 1 ? size_t(rowsB / ap->gb.G) * size_t(colsB) : 0);
  carve_adaptive(nullptr, *ap, k, nb, &ap->bytes);
  return CAFEQ_OK;
}

void fill_common(CoreParams* p, const cafeq_mat* W, const CorePlan& pl, int rep) {
  p->W = W->data; p->dtype = W->dtype; p->rows = W->rows; p->cols = W->cols; p->ld = W->ld;
  p->rep = rep; p->nseg = pl.nseg; p->nlines = pl.nlines; p->mt_per_seg = pl.mt_per_seg;
  p->n_mt = pl.n_mt; p->nwg = pl.nwg;
  p->Afwd = nullptr; p->Ainv = nullptr;
  p->do_inverse = 0; p->do_grad = 0; p->loss_kind = kLossSur; p->beta = 0.f; p->lse_t = 0.f;
  p->rG = nullptr; p->Zout = nullptr; p->codes = nullptr; p->scales = nullptr;
  p->slot_grad = nullptr; p->slot_hdr = nullptr;
  p->rec = nullptr; p->hdr_ref = nullptr; p->nslot_ref = 0; p->member_ref = nullptr;
  p->fscale = nullptr;
  p->longg = 0; p->gspan = 1; p->grec = nullptr; p->grp = 0;
  p->prep_planes = nullptr; p->prep_lscale = nullptr; p->prep_wsq = nullptr; p->fscale_inv = nullptr;
  p->prep_gtiles = nullptr;
  p->asym = 0; p->mins = nullptr; p->rec_mm = nullptr; p->grec_mm = nullptr;
  p->grid = make_grid(4);
}

// where the loss pass over prepared weights finds them
void set_prepared(CoreParams* p, const cafeq_mat* W, int axis) {
  const bool col = axis == CAFEQ_AXIS_COL;
  const PreparedLayout l = prepared_layout(col ? W->rows : W->cols, col ? W->cols : W->rows);
  const unsigned char* base = static_cast<const unsigned char*>(W->prepared);
  p->prep_wsq = reinterpret_cast<const float*>(base);
  p->prep_lscale = reinterpret_cast<const float*>(base + l.off_lscale);
  p->prep_planes = base + l.off_planes;
}

// Forward sweep(s) of the fused core over one matrix.  `p` holds everything but the group bookkeeping.  For
// groups inside a segment this is one launch.  For groups that span gspan segments: a forward-only sweep that
// records every segment's arg-max, the combination of the records per group, then the sweep proper, which
// takes each group's absmax from the combined records (both sweeps run the same kernel variant, so they see
// bit-identical transformed weights).
int run_core(int K, int axis, const GroupPlan& gp, CoreParams p, float2* rec, float2* grec, bool want_rec,
             hipStream_t st, const cafeq_mat* prepared_of = nullptr, float2* rec_mm = nullptr,
             float2* grec_mm = nullptr) {
  int rc;
  if (prepared_of) {
    // loss pass over the prepared copy of the weights
    set_prepared(&p, prepared_of, axis);
    p.rec = want_rec ? rec : nullptr;
    return launch_loss_prepared(gp.Gk, axis, p, st);
  }
  if (gp.gspan > 1) {
    CoreParams s1 = p;
    s1.do_inverse = 0; s1.do_grad = 0; s1.codes = nullptr; s1.scales = nullptr; s1.Zout = nullptr;
    s1.slot_hdr = nullptr; s1.slot_grad = nullptr; s1.rec = rec; s1.longg = 1; s1.gspan = 1; s1.grec = nullptr;
    s1.mins = nullptr; s1.rec_mm = p.asym ? rec_mm : nullptr;
    if (p.asym && (!rec_mm || !grec_mm)) return CAFEQ_ERR_INVALID_ARG;
    if ((rc = launch_core(K, gp.Gk, axis, s1, st))) return rc;
    if ((rc = launch_combine_records(rec, gp.gspan, gp.Gk, p.nlines, (p.nseg / gp.gspan), grec, st,
                                     p.asym ? rec_mm : nullptr, p.asym ? grec_mm : nullptr)))
      return rc;
    p.longg = 1; p.gspan = gp.gspan; p.grec = grec; p.rec = nullptr; p.grec_mm = p.asym ? grec_mm : nullptr;
  } else {
    p.rec = want_rec ? rec : nullptr;
  }
  return launch_core(K, gp.Gk, axis, p, st);
}

// Whether the gradient passes of a call can run with one workgroup per (matrix, block) and write the gradient in
// its final form (grad_v2.hip): prepared weights, blocks of 128, no row-blocks sharing a transform block, and
// enough blocks for most of the chip (up to four rounds of workgroups: the 27B-shaped (down, up) pair, 576 blocks,
// measured 328 us this way against 350 for the partial sums and their reduction).
bool grad_owner_eligible(const cafeq_mat* const* mats, const PassPlans* const* pps, int n, int K, int rep) {
  if (K != 128 || rep != 1) return false;
  int64_t jobs = 0;
  for (int i = 0; i < n; ++i) {
    if (!mats[i]->prepared || !pps[i]->two) return false;
    jobs += pps[i]->gpass.nseg;
  }
  const int cus = device_cu_count();
  return jobs <= 4 * int64_t(cus) && jobs * 5 >= int64_t(cus) * 3;
}
GradOwnerJob grad_owner_job(const cafeq_mat* W, int axis, const PassPlans& pp, const MemberWs& m, float* out,
                            int transpose_out) {
  const bool col = axis == CAFEQ_AXIS_COL;
  const PreparedLayout l = prepared_layout(col ? W->rows : W->cols, col ? W->cols : W->rows);
  GradOwnerJob j;
  j.gtiles = static_cast<const unsigned char*>(W->prepared) + l.off_gtiles;
  j.rec = m.grec; j.rG = m.rGreal; j.out = out;
  j.nlines = pp.gpass.nlines; j.nseg = pp.gpass.nseg; j.grp = pp.gp.G; j.transpose_out = transpose_out;
  return j;
}

// The gradient pass of the two-pass scheme over one matrix (records in, gradient partials out).
int run_grad_pass(int K, int axis, const cafeq_mat* W, int rep, const PassPlans& pp, const MemberWs& m,
                  int loss_kind, float beta, float lse_t, const float* hdr_ref, int nslot_ref, float* member_ref,
                  CoreParams* pg, hipStream_t st) {
  fill_common(pg, W, pp.gpass, rep);
  pg->loss_kind = loss_kind; pg->beta = beta; pg->lse_t = lse_t;
  pg->rG = m.rGreal; pg->slot_grad = m.slot_grad; pg->rec = m.grec; pg->grp = pp.gp.G;
  pg->hdr_ref = hdr_ref; pg->nslot_ref = nslot_ref; pg->member_ref = member_ref;
  if (W->prepared && K == 128) {
    // the prepared copy also holds the weights in the operand order of this contraction
    const bool col = axis == CAFEQ_AXIS_COL;
    const PreparedLayout l = prepared_layout(col ? W->rows : W->cols, col ? W->cols : W->rows);
    pg->prep_gtiles = static_cast<const unsigned char*>(W->prepared) + l.off_gtiles;
    return launch_grad_v2_timed(*pg, st);
  }
  return launch_grad_pass_timed(K, axis, *pg, st);
}

}  // namespace

namespace cafeq {
namespace {
// Measurement aid: the caller's table of pre-created events (cafeq_set_launch_timing); nothing is created,
// allocated or synchronised here.
cafeq_launch_timing* g_timing = nullptr;
int launch_core_raw(int K, int G, int axis, const CoreParams& p, hipStream_t st) {
  if (p.asym) {
    switch (K) {
      case 32: return launch_core_asym_k32(G, axis, p, st);
      case 64: return launch_core_asym_k64(G, axis, p, st);
      case 128: return launch_core_asym_k128(G, axis, p, st);
      case 256: return launch_core_asym_k256(G, axis, p, st);
      default: return CAFEQ_ERR_UNSUPPORTED;
    }
  }
  switch (K) {
    case 32: return launch_core_k32(G, axis, p, st);
    case 64: return launch_core_k64(G, axis, p, st);
    case 128: return launch_core_k128(G, axis, p, st);
    case 256: return launch_core_k256(G, axis, p, st);
    default: return CAFEQ_ERR_UNSUPPORTED;
  }
}
template <typename F>
int timed_launch(hipStream_t st, F&& launch, int kind = 0) {
  cafeq_launch_timing* t = g_timing;
  if (!t || t->kind != kind || t->count >= t->capacity) return launch();
  const int nth = t->seen++;
  if (t->every > 1 && nth % t->every != 0) return launch();
  const int i = t->count;
  (void)hipEventRecord(static_cast<hipEvent_t>(t->start[i]), st);
  const int rc = launch();
  (void)hipEventRecord(static_cast<hipEvent_t>(t->stop[i]), st);
  t->count = i + 1;
  return rc;
}
}  // namespace
int launch_core(int K, int G, int axis, const CoreParams& p, hipStream_t st) {
  return timed_launch(st, [&] { return launch_core_raw(K, G, axis, p, st); });
}
int launch_loss_prepared(int G, int axis, const CoreParams& p, hipStream_t st) {
  return timed_launch(st, [&] { return launch_loss_v2(G, axis, p, st); });
}
int launch_loss_prepared_pair(int G, const CoreParams& pa, const CoreParams& pb, hipStream_t st) {
  return timed_launch(st, [&] { return launch_loss_v2_pair(G, pa, pb, st); });
}
// the gradient pass over the weights, with the caller's timing events when the table asks for kind 1
int launch_grad_owner_timed(const GradOwnerJob* jobs, int n, int loss_kind, float beta, float lse_t, const double* lse_ms,
                            hipStream_t st, const LossArgs* fold) {
  return timed_launch(st, [&] { return launch_grad_v2_owner(jobs, n, loss_kind, beta, lse_t, lse_ms, st, fold); }, 1);
}
int launch_grad_v2_timed(const CoreParams& p, hipStream_t st) {
  return timed_launch(st, [&] { return launch_grad_v2(p, st); }, 1);
}
int launch_grad_pass_timed(int K, int axis, const CoreParams& p, hipStream_t st) {
  return timed_launch(st, [&] { return launch_grad_pass(K, axis, p, st); }, 1);
}
size_t core_lds_bytes(int K, int G, bool do_grad) {
  switch (K) {
    case 32: return core_lds_bytes_k32(G, do_grad);
    case 64: return core_lds_bytes_k64(G, do_grad);
    case 128: return core_lds_bytes_k128(G, do_grad);
    case 256: return core_lds_bytes_k256(G, do_grad);
    default: return 0;
  }
}
}  // namespace cafeq

namespace {
constexpr size_t kLdsLimit = 160 * 1024;
}  // namespace

extern "C" {

const char* cafeq_strerror(int status) {
  switch (status) {
    case CAFEQ_OK: return "ok";
    case CAFEQ_ERR_INVALID_ARG: return "invalid argument";
    case CAFEQ_ERR_BAD_SHAPE: return "shape not divisible as required";
    case CAFEQ_ERR_BAD_ALIGN: return "pointer or leading dimension misaligned";
    case CAFEQ_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case CAFEQ_ERR_SINGULAR: return "singular transform block";
    case CAFEQ_ERR_LAUNCH: return "HIP launch failed";
    case CAFEQ_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
  }
}

int cafeq_pqe(const float* U, const float* V, int64_t rowsA, int64_t colsA, int64_t rowsB, int64_t colsB,
              const cafeq_quant_cfg* cfg, int k, int nb, int rep, const int8_t* codesU, const float* scalesU,
              const int8_t* codesV, const float* scalesV, float* out, void* ws, void* stream) {
  int rc = check_cfg(cfg, false);
  if (rc) return rc;
  if (!U || !V || !codesU || !scalesU || !codesV || !scalesV || !out) return CAFEQ_ERR_INVALID_ARG;
  if (!supported_block(k)) return CAFEQ_ERR_UNSUPPORTED;
  if (nb <= 0 || rep <= 0 || rowsA <= 0 || colsB <= 0) return CAFEQ_ERR_BAD_SHAPE;
  if (colsA != int64_t(nb) * k || rowsB != int64_t(nb) * rep * k || colsB % 4 != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (!aligned16(U) || !aligned16(V) || !aligned16(codesU) || !aligned16(codesV) || !aligned16(scalesU) ||
      !aligned16(scalesV))
    return CAFEQ_ERR_BAD_ALIGN;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  AdaptivePlan ap;
  if ((rc = plan_adaptive(cfg, k, nb, rep, rowsA, colsA, rowsB, colsB, &ap))) return rc;
  const size_t kk = size_t(k) * k;
  Carver c(ws);
  float* partialU = c.take<float>(size_t(nb) * ap.nchunkA * 3 * kk);
  float* partialV = c.take<float>(size_t(nb) * rep * ap.nchunkB * 3 * kk);
  double* sums = c.take<double>(size_t(nb) * (1 + rep) * 3 * kk + 2 * size_t(nb) * rep);
  return launch_pqe(U, V, rowsA, colsA, rowsB, colsB, k, ap.ga.G, ap.gb.G, nb, rep, codesU, scalesU, codesV, scalesV,
                    ap.chunkA, ap.nchunkA, ap.chunkB, ap.nchunkB, partialU, partialV, sums, out,
                    static_cast<hipStream_t>(stream));
}

int cafeq_version(void) { return 100; }

namespace {
struct OptWs { float* grad; void* orth; void* sub; };
OptWs carve_opt(void* ws, int k, int nb) {
  char* base = static_cast<char*>(ws);
  OptWs w;
  w.grad = reinterpret_cast<float*>(base);
  w.orth = base + align_up(size_t(nb) * k * k * sizeof(float), 256);
  w.sub = static_cast<char*>(w.orth) + orth_ws_any(k, nb);
  return w;
}
// The inverse of iteration s of a learning loop: from scratch first, then warm-started from the previous one.
int loop_inverse(int s, const float* T, int k, int nb, float* Tinv, int* status, void* ws, void* stream) {
  if (s == 0 || (k != 64 && k != 128 && k != 256)) return cafeq_block_inverse(T, k, nb, Tinv, nullptr, nullptr, status, ws, stream);
  return launch_block_inverse_warm(T, k, nb, static_cast<double*>(ws), Tinv, status, static_cast<hipStream_t>(stream));
}
int check_opt(const cafeq_opt_cfg* opt) {
  if (!opt) return CAFEQ_ERR_INVALID_ARG;
  if (opt->steps < 0 || !(opt->lr >= 0.f) || !(opt->lambda_orth >= 0.f)) return CAFEQ_ERR_INVALID_ARG;
  return CAFEQ_OK;
}
}  // namespace

static int dual_impl(const cafeq_mat* A, const cafeq_mat* B, const cafeq_xform* x, const cafeq_quant_cfg* cfg,
                     float lse_t, float* losses, float* gradT, int8_t* codesU, float* scalesU, int8_t* codesV,
                     float* scalesV, void* ws, void* stream, const AdamHook* adam);

int cafeq_optimize_single(const cafeq_mat* W, float* T, float* Tinv, int k, int nb, int rep,
                          const cafeq_quant_cfg* cfg, const cafeq_opt_cfg* opt, float* history, int* status,
                          void* ws, void* stream) {
  int rc = check_opt(opt);
  if (rc) return rc;
  if (!T || !Tinv || !history) return CAFEQ_ERR_INVALID_ARG;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const OptWs w = carve_opt(ws, k, nb);
  const int64_t n = int64_t(nb) * k * k;
  cafeq_xform x{T, Tinv, k, nb, rep};
  if ((rc = launch_fill(history, 0.f, int64_t(opt->steps) * 8, st))) return rc;
  for (int s = 0; s < opt->steps; ++s) {
    float* h = history + size_t(s) * 8;
    if ((rc = loop_inverse(s, T, k, nb, Tinv, status, w.sub, stream))) return rc;
    if ((rc = cafeq_proxy_loss_fwd_bwd(W, &x, cfg, h, w.grad, nullptr, nullptr, w.sub, stream))) return rc;
    // surrogate / ||W||^2 (history[s][2]) when normalised, then the regulariser's gradient on top
    if (opt->normalize && (rc = launch_div_by_device_scalar(w.grad, h + 2, n, st))) return rc;
    if (opt->lambda_orth > 0.f &&
        (rc = cafeq_orth_penalty(T, k, nb, opt->lambda_orth, h + 4, w.grad, w.orth, stream)))
      return rc;
    if ((rc = cafeq_sgd_update(T, w.grad, opt->lr, nullptr, n, stream))) return rc;
  }
  return cafeq_block_inverse(T, k, nb, Tinv, nullptr, nullptr, status, w.sub, stream);
}

int cafeq_optimize_pair(const cafeq_mat* A, const cafeq_mat* B, float* T, float* Tinv, int k, int nb, int rep,
                        const cafeq_quant_cfg* cfg, float lse_t, const cafeq_opt_cfg* opt, float* moments,
                        float* history, int* status, void* ws, void* stream) {
  int rc = check_opt(opt);
  if (rc) return rc;
  if (!T || !Tinv || !history || !moments) return CAFEQ_ERR_INVALID_ARG;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const OptWs w = carve_opt(ws, k, nb);
  const int64_t n = int64_t(nb) * k * k;
  cafeq_xform x{T, Tinv, k, nb, rep};
  if ((rc = launch_fill(history, 0.f, int64_t(opt->steps) * 8, st))) return rc;
  if ((rc = launch_fill(moments, 0.f, 2 * n, st))) return rc;
  const bool fuse_adam = !(opt->lambda_orth > 0.f) && (k == 64 || k == 128 || k == 256);
  for (int s = 0; s < opt->steps; ++s) {
    float* h = history + size_t(s) * 8;
    if ((rc = loop_inverse(s, T, k, nb, Tinv, status, w.sub, stream))) return rc;
    if (fuse_adam) {
      // the Adam step rides in the epilogue of the gradient's last kernel (no regulariser to add in between)
      if (!(opt->beta1 >= 0.0 && opt->beta1 < 1.0 && opt->beta2 >= 0.0 && opt->beta2 < 1.0)) return CAFEQ_ERR_INVALID_ARG;
      AdamHook hook;
      hook.T = T; hook.m = moments; hook.v = moments + n;
      hook.lr = float(opt->lr); hook.beta1 = float(opt->beta1); hook.omb1 = float(1.0 - opt->beta1);
      hook.beta2 = float(opt->beta2); hook.omb2 = float(1.0 - opt->beta2); hook.eps = float(opt->eps);
      hook.c1 = float(1.0 / (1.0 - pow(opt->beta1, double(s + 1))));
      hook.c2 = float(1.0 / (1.0 - pow(opt->beta2, double(s + 1))));
      if ((rc = dual_impl(A, B, &x, cfg, lse_t, h, w.grad, nullptr, nullptr, nullptr, nullptr, w.sub, stream, &hook)))
        return rc;
      continue;
    }
    if ((rc = cafeq_dual_proxy_loss_fwd_bwd(A, B, &x, cfg, lse_t, h, w.grad, nullptr, nullptr, nullptr, nullptr, w.sub,
                                            stream)))
      return rc;
    if (opt->lambda_orth > 0.f &&
        (rc = cafeq_orth_penalty(T, k, nb, opt->lambda_orth, h + 6, w.grad, w.orth, stream)))
      return rc;
    if ((rc = cafeq_adam_update(T, w.grad, moments, moments + n, s + 1, opt->lr, opt->beta1, opt->beta2, opt->eps, n,
                                stream)))
      return rc;
  }
  return cafeq_block_inverse(T, k, nb, Tinv, nullptr, nullptr, status, w.sub, stream);
}


namespace cafeq {
namespace {
__global__ __launch_bounds__(256) void stream_read_kernel(const uintx4* __restrict__ p, size_t n16, unsigned* sink) {
  unsigned acc = 0;
  const size_t stride = size_t(gridDim.x) * 1024;
  size_t base = size_t(blockIdx.x) * 1024 + threadIdx.x;
  for (; base + 768 < n16; base += stride) {
    uintx4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(p + base + 256 * u);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {       // the last, partial step of 1024 vectors (every later step lies beyond the end)
    const size_t i = base + 256 * u;
    if (i < n16) {
      const uintx4 v = p[i];
      acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
  }
  if (acc == 0x5EEDF00Du) sink[0] = acc;
}
}  // namespace
}  // namespace cafeq

int cafeq_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink || bytes < 16 || bytes % 16 != 0 || reinterpret_cast<uintptr_t>(buf) % 16 != 0) return CAFEQ_ERR_INVALID_ARG;
  const size_t n16 = bytes / 16;
  const size_t steps = (n16 + 1023) / 1024;
  const unsigned grid = unsigned(std::min<size_t>(steps, 8192));
  hipLaunchKernelGGL(cafeq::stream_read_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const cafeq::uintx4*>(buf), n16, static_cast<unsigned*>(sink));
  CAFEQ_CHECK_LAUNCH();
  return CAFEQ_OK;
}

int cafeq_set_launch_timing(cafeq_launch_timing* t) {
  if (t && (t->capacity < 0 || t->count < 0 || (t->capacity > 0 && (!t->start || !t->stop)))) return CAFEQ_ERR_INVALID_ARG;
  cafeq::g_timing = t;
  return CAFEQ_OK;
}

size_t cafeq_workspace_bytes(int call_id, const cafeq_mat* a, const cafeq_mat* b, const cafeq_xform* x,
                             const cafeq_quant_cfg* cfg) {
  if (x && small_m(x->k) && call_id != CAFEQ_CALL_ORTH_PENALTY && call_id != CAFEQ_CALL_OPTIMIZE_SINGLE &&
      call_id != CAFEQ_CALL_OPTIMIZE_PAIR) {
    // blocks smaller than 32: the embedding's scratch in front of what the same call needs with blocks of 32
    int64_t nb32 = 0;
    switch (call_id) {
      case CAFEQ_CALL_PROXY_LOSS:
        if (!a || !cfg) return 0;
        nb32 = small_nb32(x, cfg->axis == CAFEQ_AXIS_COL ? a->cols : a->rows);
        break;
      case CAFEQ_CALL_DUAL_PROXY_LOSS:
        if (!a || x->rep != 1) return 0;
        nb32 = small_nb32(x, a->cols);
        break;
      case CAFEQ_CALL_APPLY_TRANSFORM:
      case CAFEQ_CALL_BLOCK_INVERSE:
        nb32 = (int64_t(x->nb) * (x->rep > 0 ? x->rep : 1) * x->k) / 32;
        if (nb32 * 32 != int64_t(x->nb) * (x->rep > 0 ? x->rep : 1) * x->k) nb32 = 0;
        break;
      default: return 0;   // Alg. 1 and the paired error work per head: blocks of 32 and more
    }
    if (nb32 <= 0 || nb32 > (int64_t(1) << 30)) return 0;
    const cafeq_xform x32{nullptr, nullptr, 32, int(nb32), 1};
    const size_t sub = cafeq_workspace_bytes(call_id, a, b, &x32, cfg);
    return sub ? carve_small(nullptr, nb32).head + sub : 0;
  }
  switch (call_id) {
    case CAFEQ_CALL_RTN_QUANTIZE:
      if (!a) return 0;
      return align_up(rtn_partials_capacity(a->rows, a->cols) * sizeof(double), 256);
    case CAFEQ_CALL_APPLY_TRANSFORM:
      if (!x) return 0;
      return align_up(size_t(x->nb) * kFwdPlanes * x->k * x->k * sizeof(uint16_t), 256);
    case CAFEQ_CALL_BLOCK_INVERSE:
      if (!x) return 0;
      return align_up(size_t(x->nb) * x->k * 2 * x->k * sizeof(double), 256);
    case CAFEQ_CALL_PROXY_LOSS: {
      if (!a || !x || !cfg) return 0;
      const bool col = cfg->axis == CAFEQ_AXIS_COL;
      const int64_t naxis = col ? a->cols : a->rows, nlines = col ? a->rows : a->cols;
      GroupPlan gp;
      if (resolve_group(cfg, naxis, x->k, &gp)) return 0;
      PassPlans pg, pn;
      const bool mm = is_minmax(cfg);
      if (plan_passes(x->k, gp, nlines, naxis, false, &pn, false, mm)) return 0;
      size_t bytes = carve_single(nullptr, pn, x->nb, false).bytes;
      // (where the gradient has no kernel the forward-only size is still reported)
      if (!plan_passes(x->k, gp, nlines, naxis, true, &pg, false, mm)) bytes = std::max(bytes, carve_single(nullptr, pg, x->nb, true).bytes);
      return bytes;
    }
    case CAFEQ_CALL_DUAL_PROXY_LOSS: {
      if (!a || !b || !x || !cfg) return 0;
      GroupPlan ga, gb;
      if (resolve_group(cfg, a->cols, x->k, &ga) || resolve_group(cfg, b->rows, x->k, &gb)) return 0;
      PassPlans qa, qb, na, nbp;
      const bool mm = is_minmax(cfg);
      if (plan_passes(x->k, ga, a->rows, a->cols, false, &na, false, mm) ||
          plan_passes(x->k, gb, b->cols, b->rows, false, &nbp, false, mm))
        return 0;
      size_t bytes = carve_dual(nullptr, na, nbp, x->nb, false).bytes;
      if (!plan_passes(x->k, ga, a->rows, a->cols, true, &qa, false, mm) &&
          !plan_passes(x->k, gb, b->cols, b->rows, true, &qb, false, mm))
        bytes = std::max(bytes, carve_dual(nullptr, qa, qb, x->nb, true).bytes);
      return bytes;
    }
    case CAFEQ_CALL_ORTH_PENALTY:
      if (!x) return 0;
      return orth_ws_any(x->k, x->nb);
    case CAFEQ_CALL_OPTIMIZE_SINGLE:
    case CAFEQ_CALL_OPTIMIZE_PAIR: {
      // gradient buffer + regulariser scratch + the larger of the sub-calls' workspaces
      if (!x) return 0;
      const size_t sub = std::max(
          cafeq_workspace_bytes(call_id == CAFEQ_CALL_OPTIMIZE_SINGLE ? CAFEQ_CALL_PROXY_LOSS : CAFEQ_CALL_DUAL_PROXY_LOSS,
                                a, b, x, cfg),
          cafeq_workspace_bytes(CAFEQ_CALL_BLOCK_INVERSE, a, b, x, cfg));
      if (sub == 0) return 0;
      return align_up(size_t(x->nb) * x->k * x->k * sizeof(float), 256) + orth_ws_any(x->k, x->nb) + sub;
    }
    case CAFEQ_CALL_PQE: {
      if (!a || !b || !x || !cfg) return 0;
      AdaptivePlan ap;
      if (plan_adaptive(cfg, x->k, x->nb, x->rep, a->rows, a->cols, b->rows, b->cols, &ap)) return 0;
      const size_t kk = size_t(x->k) * x->k;
      Carver c(nullptr);
      c.take<float>(size_t(x->nb) * ap.nchunkA * 3 * kk);
      c.take<float>(size_t(x->nb) * x->rep * ap.nchunkB * 3 * kk);
      c.take<double>(size_t(x->nb) * (1 + x->rep) * 3 * kk + 2 * size_t(x->nb) * x->rep);
      return c.off;
    }
    case CAFEQ_CALL_ADAPTIVE_ROUND: {
      // a: U [rowsA][nb*k], b: V [nb*rep*k][colsB]
      if (!a || !b || !x || !cfg) return 0;
      AdaptivePlan ap;
      if (plan_adaptive(cfg, x->k, x->nb, x->rep, a->rows, a->cols, b->rows, b->cols, &ap)) return 0;
      return ap.bytes;
    }
    default:
      return 0;
  }
}

size_t cafeq_prepared_bytes(const cafeq_mat* W, int axis) {
  if (!W || W->rows <= 0 || W->cols <= 0 || (axis != CAFEQ_AXIS_COL && axis != CAFEQ_AXIS_ROW)) return 0;
  const bool col = axis == CAFEQ_AXIS_COL;
  const int64_t nlines = col ? W->rows : W->cols, naxis = col ? W->cols : W->rows;
  if (naxis % 128 != 0) return 0;
  return prepared_layout(nlines, naxis).bytes;
}

int cafeq_prepare_weights(const cafeq_mat* W, int axis, void* prepared, void* stream) {
  int rc = check_mat(W);
  if (rc) return rc;
  if (axis != CAFEQ_AXIS_COL && axis != CAFEQ_AXIS_ROW) return CAFEQ_ERR_INVALID_ARG;
  if (!prepared) return CAFEQ_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(prepared) & 255u) != 0) return CAFEQ_ERR_BAD_ALIGN;
  return launch_prepare(W, axis, prepared, static_cast<hipStream_t>(stream));
}

int cafeq_rtn_quantize(const cafeq_mat* W, const cafeq_quant_cfg* cfg, int8_t* codes, float* scales,
                       float* err_sq, void* ws, void* stream) {
  int rc = check_mat(W);
  if (rc) return rc;
  rc = check_cfg(cfg, true);
  if (rc) return rc;
  if (!codes) return CAFEQ_ERR_INVALID_ARG;
  if (!aligned16(codes) || (scales && !aligned16(scales))) return CAFEQ_ERR_BAD_ALIGN;
  const int64_t line = cfg->axis == CAFEQ_AXIS_COL ? W->cols : W->rows;
  const int64_t g = cfg->group == 0 ? line : cfg->group;
  if (line % g != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (err_sq && !ws) return CAFEQ_ERR_WORKSPACE;
  RtnArgs a;
  a.W = W->data; a.dtype = W->dtype; a.rows = W->rows; a.cols = W->cols; a.ld = W->ld;
  a.axis = cfg->axis; a.group = cfg->group; a.grid = make_grid(cfg->bits);
  a.codes = codes; a.scales = scales; a.mins = nullptr;
  a.partial = err_sq ? static_cast<double*>(ws) : nullptr;
  a.err_sq = err_sq;
  return launch_rtn(a, static_cast<hipStream_t>(stream));
}

int cafeq_rtn_quantize_minmax(const cafeq_mat* W, const cafeq_quant_cfg* cfg, uint8_t* codes, float* scales,
                              float* mins, float* err_sq, void* ws, void* stream) {
  int rc = check_mat(W);
  if (rc) return rc;
  if (!cfg || cfg->bits < 1 || cfg->bits > 8 || cfg->group < 0) return CAFEQ_ERR_INVALID_ARG;
  if (cfg->axis != CAFEQ_AXIS_COL && cfg->axis != CAFEQ_AXIS_ROW) return CAFEQ_ERR_INVALID_ARG;
  if (!codes) return CAFEQ_ERR_INVALID_ARG;
  if (!aligned16(codes) || (scales && !aligned16(scales)) || (mins && !aligned16(mins))) return CAFEQ_ERR_BAD_ALIGN;
  const int64_t line = cfg->axis == CAFEQ_AXIS_COL ? W->cols : W->rows;
  const int64_t g = cfg->group == 0 ? line : cfg->group;
  if (line % g != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (err_sq && !ws) return CAFEQ_ERR_WORKSPACE;
  RtnArgs a;
  a.W = W->data; a.dtype = W->dtype; a.rows = W->rows; a.cols = W->cols; a.ld = W->ld;
  a.axis = cfg->axis; a.group = cfg->group; a.grid = make_grid(2);
  a.codes = reinterpret_cast<int8_t*>(codes); a.scales = scales; a.mins = mins;
  a.partial = err_sq ? static_cast<double*>(ws) : nullptr;
  a.err_sq = err_sq;
  return launch_rtn_minmax(a, cfg->bits, static_cast<hipStream_t>(stream));
}

int cafeq_block_inverse(const float* T, int k, int nb, float* Tinv, float* rho_row, float* rho_col,
                        int* status, void* ws, void* stream) {
  if (!T || !Tinv) return CAFEQ_ERR_INVALID_ARG;
  if (nb < 1) return CAFEQ_ERR_BAD_SHAPE;
  if (const int m = small_m(k)) {
    // a run of 32 / k blocks as one block-diagonal block of 32 (its inverse is block-diagonal too; the squared
    // row / column norms keep their positions; a singular block marks its whole run)
    if (nb % m != 0) return CAFEQ_ERR_BAD_SHAPE;
    if (!ws) return CAFEQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nb32 = nb / m;
    const SmallWs w = carve_small(ws, nb32);
    int rc;
    if ((rc = launch_embed_blocks(T, k, nb, 1, nb32, w.T32, st))) return rc;
    if ((rc = cafeq_block_inverse(w.T32, 32, nb32, w.P32, rho_row, rho_col, status ? w.st32 : nullptr, w.sub, stream)))
      return rc;
    if ((rc = launch_gather_blocks(w.P32, k, nb, 1, Tinv, st))) return rc;
    if (status && (rc = launch_expand_status(w.st32, m, nb, status, st))) return rc;
    return CAFEQ_OK;
  }
  if (k != 32 && k != 64 && k != 128 && k != 256) return CAFEQ_ERR_UNSUPPORTED;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  return launch_block_inverse(T, k, nb, static_cast<double*>(ws), Tinv, rho_row, rho_col, status,
                              static_cast<hipStream_t>(stream));
}

int cafeq_apply_transform(const cafeq_mat* W, const cafeq_xform* x, int axis, int side, float* Z,
                          void* ws, void* stream) {
  int rc = check_mat(W);
  if (rc) return rc;
  if (side != CAFEQ_SIDE_T && side != CAFEQ_SIDE_TINV) return CAFEQ_ERR_INVALID_ARG;
  if (x && small_m(x->k)) {
    if ((rc = check_small_xform(x, side == CAFEQ_SIDE_TINV))) return rc;
    if ((rc = check_axis_len(W, x, axis))) return rc;
    if (!ws) return CAFEQ_ERR_WORKSPACE;
    const int64_t nb32 = small_nb32(x, axis == CAFEQ_AXIS_COL ? W->cols : W->rows);
    if (nb32 <= 0) return CAFEQ_ERR_BAD_SHAPE;
    const SmallWs w = carve_small(ws, nb32);
    if ((rc = launch_embed_blocks(side == CAFEQ_SIDE_T ? x->T : x->Tinv, x->k, x->nb, x->rep, int(nb32), w.T32,
                                  static_cast<hipStream_t>(stream))))
      return rc;
    const cafeq_xform x32{w.T32, w.T32, 32, int(nb32), 1};
    return cafeq_apply_transform(W, &x32, axis, side, Z, w.sub, stream);
  }
  rc = check_xform(x, side == CAFEQ_SIDE_TINV);
  if (rc) return rc;
  rc = check_axis_len(W, x, axis);
  if (rc) return rc;
  if (!Z) return CAFEQ_ERR_INVALID_ARG;
  if (!aligned16(Z)) return CAFEQ_ERR_BAD_ALIGN;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  const bool col = axis == CAFEQ_AXIS_COL;
  CorePlan pl;
  rc = make_plan(x->k, x->k, col ? W->rows : W->cols, col ? W->cols : W->rows, &pl, false);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* planes = static_cast<uint16_t*>(ws);
  // half-precision forward operands where the kernel variant exists: two planes, and the per-block factors
  // in the room of the third
  float* fs = core_forward_f16(x->k, x->k, 4) ? reinterpret_cast<float*>(planes + size_t(x->nb) * 2 * x->k * x->k) : nullptr;
  {
    const SplitRequest req{side == CAFEQ_SIDE_T ? x->T : x->Tinv, planes, col ? 1 : 0, kFwdPlanes, fs};
    if ((rc = launch_split_planes_multi(&req, 1, x->k, x->nb, st))) return rc;
  }
  CoreParams p;
  fill_common(&p, W, pl, x->rep);
  p.Afwd = planes; p.Ainv = nullptr; p.fscale = fs;
  p.Zout = Z;
  return launch_core(x->k, x->k, axis, p, st);
}

int cafeq_proxy_loss_fwd_bwd(const cafeq_mat* W, const cafeq_xform* x, const cafeq_quant_cfg* cfg,
                             float* losses, float* gradT, int8_t* codes, float* scales, void* ws,
                             void* stream) {
  int rc = check_mat(W);
  if (rc) return rc;
  rc = check_cfg(cfg, true, true);
  if (rc) return rc;
  if (x && small_m(x->k)) {
    if ((rc = check_small_xform(x, true))) return rc;
    if ((rc = check_axis_len(W, x, cfg->axis))) return rc;
    if (!ws) return CAFEQ_ERR_WORKSPACE;
    if (gradT && !aligned16(gradT)) return CAFEQ_ERR_BAD_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nb32 = small_nb32(x, cfg->axis == CAFEQ_AXIS_COL ? W->cols : W->rows);
    if (nb32 <= 0) return CAFEQ_ERR_BAD_SHAPE;
    const SmallWs w = carve_small(ws, nb32);
    if ((rc = launch_embed_blocks(x->T, x->k, x->nb, x->rep, int(nb32), w.T32, st))) return rc;
    if ((rc = launch_embed_blocks(x->Tinv, x->k, x->nb, x->rep, int(nb32), w.P32, st))) return rc;
    const cafeq_xform x32{w.T32, w.P32, 32, int(nb32), 1};
    if ((rc = cafeq_proxy_loss_fwd_bwd(W, &x32, cfg, losses, gradT ? w.G32 : nullptr, codes, scales, w.sub, stream)))
      return rc;
    return gradT ? launch_gather_blocks(w.G32, x->k, x->nb, x->rep, gradT, st) : CAFEQ_OK;
  }
  rc = check_xform(x, true);
  if (rc) return rc;
  rc = check_axis_len(W, x, cfg->axis);
  if (rc) return rc;
  if (!losses) return CAFEQ_ERR_INVALID_ARG;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  if ((codes && !aligned16(codes)) || (scales && !aligned16(scales)) || (gradT && !aligned16(gradT)))
    return CAFEQ_ERR_BAD_ALIGN;
  const bool col = cfg->axis == CAFEQ_AXIS_COL;
  const int64_t naxis = col ? W->cols : W->rows, nlines = col ? W->rows : W->cols;
  const int K = x->k, nb = x->nb;
  GroupPlan gp;
  rc = resolve_group(cfg, naxis, K, &gp);
  if (rc) return rc;
  const bool grad = gradT != nullptr;
  const bool asym = is_minmax(cfg);
  const bool v2 = v2_eligible(W, K, gp, cfg);
  PassPlans pp;
  rc = plan_passes(K, gp, nlines, naxis, grad, &pp, v2, asym);
  if (rc) return rc;
  const CorePlan& pl = pp.first;
  {
    const size_t lds = core_lds_bytes(K, gp.Gk, pp.fused);
    if (lds == 0 || lds > kLdsLimit) return CAFEQ_ERR_UNSUPPORTED;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  SingleWs w = carve_single(ws, pp, nb, grad);
  const QGrid grid = grid_for(cfg);
  const float beta = beta_for(cfg, grid);
  const bool f16 = !asym && core_forward_f16(K, gp.Gk, cfg->bits);

  // rho per axis index, its sums per segment-level group (the loss sweep) and per group (the gradient pass)
  // (groups inside a block, or of a few whole blocks: the same launch)
  const bool rg_inline = rho_groups_inline(K, nb, gp.Gk, x->rep);
  if ((rc = launch_rho(x->Tinv, K, nb, col ? 1 : 0, w.rho, st, rg_inline ? w.m.rG : nullptr, gp.Gk, x->rep))) return rc;
  if (!rg_inline && (rc = launch_rho_groups(w.rho, K, x->rep, gp.Gk, naxis / gp.Gk, w.m.rG, st))) return rc;
  if (gp.gspan > 1 && (rc = launch_rho_groups(w.rho, K, x->rep, gp.G, naxis / gp.G, w.m.rGreal, st))) return rc;

  CoreParams p;
  fill_common(&p, W, pl, x->rep);
  // forward operand [out][in]: T^T (COL) or T (ROW); inverse operand: Tinv^T or Tinv
  {
    // (prepared weights: float16 planes for both operands, scaled so that the rounding error fits float16)
    const SplitRequest req[2] = {{x->T, w.m.pfwd, col ? 1 : 0, kFwdPlanes, f16 ? w.m.fs : nullptr, v2 ? 1 : 0, v2 ? 4 : 14},
                                 {x->Tinv, w.m.pinv, col ? 1 : 0, kInvPlanes, v2 ? w.m.fsi : nullptr, 0, 4}};
    if ((rc = launch_split_planes_multi(req, 2, K, nb, st, w.slot_hdr, pl.nslot))) return rc;
  }
  p.Afwd = w.m.pfwd; p.Ainv = w.m.pinv; p.fscale = f16 ? w.m.fs : nullptr; p.fscale_inv = v2 ? w.m.fsi : nullptr;
  p.grid = grid; p.do_inverse = 1; p.do_grad = pp.fused ? 1 : 0; p.loss_kind = kLossSur; p.beta = beta;
  p.rG = w.m.rG; p.codes = codes; p.scales = scales; p.slot_grad = w.m.slot_grad; p.slot_hdr = w.slot_hdr;
  p.asym = asym ? 1 : 0;
  p.mins = asym && scales ? scales + nlines * (naxis / gp.G) : nullptr;   // the minima follow the scales
  if ((rc = run_core(K, cfg->axis, gp, p, w.m.rec, w.m.grec, pp.two, st, v2 ? W : nullptr, w.m.rec_mm, w.m.grec_mm)))
    return rc;
  const cafeq_mat* mats[1] = {W};
  const PassPlans* pps[1] = {&pp};
  const bool owner = grad && grad_owner_eligible(mats, pps, 1, K, x->rep);
  // (with one workgroup per block in the gradient pass, its first workgroup reduces the losses: one launch less)
  // (with gradient partials, the loss reduction rides in the launch that reduces them)
  if (!grad && (rc = launch_reduce_losses(kLossSur, w.slot_hdr, int(pl.nslot), nullptr, 0, beta, 0.f, 0, losses,
                                          w.lse_ms, st)))
    return rc;
  if (grad) {
    // path through Z (fused into the pass above, or a second pass over the weights from its
    // arg-max records), then the path through rho(P): -2 P^T Mmid P^T
    CoreParams pg = p;
    if (owner) {
      const GradOwnerJob job = grad_owner_job(W, cfg->axis, pp, w.m, gradT, col ? 1 : 0);
      LossArgs la{};
      la.hdrA = w.slot_hdr; la.nslotA = int(pl.nslot); la.kind = kLossSur; la.beta = beta; la.losses = losses;
      la.lse_ms = w.lse_ms;
      if ((rc = launch_grad_owner_timed(&job, 1, kLossSur, beta, 0.f, nullptr, st, &la))) return rc;
    } else {
      if (pp.two &&
          (rc = run_grad_pass(K, cfg->axis, W, x->rep, pp, w.m, kLossSur, beta, 0.f, nullptr, 0, nullptr, &pg, st)))
        return rc;
      // gradient reduction, the middle factor of the rho path and the loss reduction in one launch
      if ((rc = launch_single_tail(pg, p, K, gp.Gk, pp.fused, nb, col ? 1 : 0, gradT, x->Tinv, col ? 1 : 0, w.mmid, beta,
                                   int(pl.nslot), losses, w.lse_ms, st)))
        return rc;
    }
    if (owner && (rc = launch_build_mmid(p, K, gp.Gk, nb, x->Tinv, col ? 1 : 0, w.mmid, st))) return rc;
    if ((rc = launch_bgemm_chain(x->Tinv, w.mmid, w.x1, gradT, K, nb, -2.f, 1.f, st))) return rc;
  }
  return CAFEQ_OK;
}

// adam (learning loop only; blocks of 64 and more): the last kernel of the gradient applies the Adam step to T, m
// and v instead of storing the gradient (gradT is then scratch)
static int dual_impl(const cafeq_mat* A, const cafeq_mat* B, const cafeq_xform* x, const cafeq_quant_cfg* cfg,
                     float lse_t, float* losses, float* gradT, int8_t* codesU, float* scalesU, int8_t* codesV,
                     float* scalesV, void* ws, void* stream, const AdamHook* adam) {
  int rc = check_mat(A);
  if (rc) return rc;
  rc = check_mat(B);
  if (rc) return rc;
  rc = check_cfg(cfg, false, true);
  if (rc) return rc;
  if (x && small_m(x->k)) {
    // (row-blocks that share a small block do not line up with blocks of 32: rep must be 1 here)
    if (adam) return CAFEQ_ERR_INVALID_ARG;
    if ((rc = check_small_xform(x, true))) return rc;
    if (x->rep != 1) return CAFEQ_ERR_UNSUPPORTED;
    if (A->cols != int64_t(x->nb) * x->k || B->rows != A->cols) return CAFEQ_ERR_BAD_SHAPE;
    if (!ws) return CAFEQ_ERR_WORKSPACE;
    if (gradT && !aligned16(gradT)) return CAFEQ_ERR_BAD_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nb32 = small_nb32(x, A->cols);
    if (nb32 <= 0) return CAFEQ_ERR_BAD_SHAPE;
    const SmallWs w = carve_small(ws, nb32);
    if ((rc = launch_embed_blocks(x->T, x->k, x->nb, 1, int(nb32), w.T32, st))) return rc;
    if ((rc = launch_embed_blocks(x->Tinv, x->k, x->nb, 1, int(nb32), w.P32, st))) return rc;
    const cafeq_xform x32{w.T32, w.P32, 32, int(nb32), 1};
    if ((rc = cafeq_dual_proxy_loss_fwd_bwd(A, B, &x32, cfg, lse_t, losses, gradT ? w.G32 : nullptr, codesU, scalesU,
                                            codesV, scalesV, w.sub, stream)))
      return rc;
    return gradT ? launch_gather_blocks(w.G32, x->k, x->nb, 1, gradT, st) : CAFEQ_OK;
  }
  rc = check_xform(x, true);
  if (rc) return rc;
  if (!losses) return CAFEQ_ERR_INVALID_ARG;
  if (!(lse_t > 0.f)) return CAFEQ_ERR_INVALID_ARG;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  const int K = x->k, nb = x->nb;
  if (A->cols != int64_t(nb) * K || B->rows != int64_t(nb) * x->rep * K) return CAFEQ_ERR_BAD_SHAPE;
  GroupPlan ga, gb;
  if ((rc = resolve_group(cfg, A->cols, K, &ga))) return rc;
  if ((rc = resolve_group(cfg, B->rows, K, &gb))) return rc;
  const bool grad = gradT != nullptr;
  const bool asym = is_minmax(cfg);
  const bool v2A = v2_eligible(A, K, ga, cfg), v2B = v2_eligible(B, K, gb, cfg);
  // both loss passes over prepared weights in one launch, each member on half of the chip: when neither writes
  // codes or scales and both use the same group length
  const bool pair_launch = v2A && v2B && !codesU && !scalesU && !codesV && !scalesV && ga.Gk == gb.Gk;
  PassPlans qa, qb;
  if ((rc = plan_passes(K, ga, A->rows, A->cols, grad, &qa, v2A, asym, pair_launch ? 2 : 1))) return rc;
  if ((rc = plan_passes(K, gb, B->cols, B->rows, grad, &qb, v2B, asym, pair_launch ? 2 : 1))) return rc;
  const CorePlan &pa = qa.first, &pb = qb.first;
  {
    const size_t la = core_lds_bytes(K, ga.Gk, qa.fused), lb = core_lds_bytes(K, gb.Gk, qb.fused);
    if (la == 0 || lb == 0 || la > kLdsLimit || lb > kLdsLimit) return CAFEQ_ERR_UNSUPPORTED;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  DualWs w = carve_dual(ws, qa, qb, nb, grad);
  const QGrid grid = grid_for(cfg);
  // the gradient-free pass over 128 x 128 blocks (one block per segment) takes half-precision forward operands
  const bool f16A = !asym && core_forward_f16(K, ga.Gk, cfg->bits), f16B = !asym && core_forward_f16(K, gb.Gk, cfg->bits);

  {
    const SplitRequest req[4] = {{x->T, w.a.pfwd, 1, kFwdPlanes, f16A ? w.a.fs : nullptr, v2A ? 1 : 0, v2A ? 4 : 14},
                                 {x->Tinv, w.a.pinv, 1, kInvPlanes, v2A ? w.a.fsi : nullptr, 0, 4},
                                 {x->Tinv, w.b.pfwd, 0, kFwdPlanes, f16B ? w.b.fs : nullptr, v2B ? 1 : 0, v2B ? 4 : 14},
                                 {x->T, w.b.pinv, 0, kInvPlanes, v2B ? w.b.fsi : nullptr, 0, 4}};
    if ((rc = launch_split_planes_multi(req, 4, K, nb, st, w.hdrA, pa.nslot + pb.nslot))) return rc;
  }
  // Each member: the loss pass, then (two-pass gradient) straight away the gradient pass over
  // the same weights, while they are still in the memory-side cache.  The gradient pass takes
  // its exponentials relative to the member's own largest group maximum; the final reduction
  // rescales to the pair's.
  CoreParams a, ag, b, bg;
  fill_common(&a, A, pa, 1);
  a.Afwd = w.a.pfwd; a.Ainv = w.a.pinv;
  a.grid = grid; a.do_inverse = 1; a.do_grad = qa.fused ? 1 : 0; a.loss_kind = kLossLse; a.lse_t = lse_t;
  a.codes = codesU; a.scales = scalesU; a.slot_grad = w.a.slot_grad; a.slot_hdr = w.hdrA;
  a.fscale = f16A ? w.a.fs : nullptr; a.fscale_inv = v2A ? w.a.fsi : nullptr;
  a.asym = asym ? 1 : 0;
  a.mins = asym && scalesU ? scalesU + A->rows * (A->cols / ga.G) : nullptr;   // the minima follow the scales
  fill_common(&b, B, pb, x->rep);
  b.Afwd = w.b.pfwd; b.Ainv = w.b.pinv;
  b.grid = grid; b.do_inverse = 1; b.do_grad = qb.fused ? 1 : 0; b.loss_kind = kLossLse; b.lse_t = lse_t;
  b.codes = codesV; b.scales = scalesV; b.slot_grad = w.b.slot_grad; b.slot_hdr = w.hdrB;
  b.fscale = f16B ? w.b.fs : nullptr; b.fscale_inv = v2B ? w.b.fsi : nullptr;
  b.asym = asym ? 1 : 0;
  b.mins = asym && scalesV ? scalesV + (B->rows / gb.G) * B->cols : nullptr;
  const cafeq_mat* mats[2] = {A, B};
  const PassPlans* pps[2] = {&qa, &qb};
  const bool owner = grad && grad_owner_eligible(mats, pps, 2, K, x->rep);

  if (pair_launch) {
    set_prepared(&a, A, CAFEQ_AXIS_COL);
    set_prepared(&b, B, CAFEQ_AXIS_ROW);
    a.rec = qa.two ? w.a.rec : nullptr;
    b.rec = qb.two ? w.b.rec : nullptr;
    if ((rc = launch_loss_prepared_pair(ga.Gk, a, b, st))) return rc;
  } else if ((rc = run_core(K, CAFEQ_AXIS_COL, ga, a, w.a.rec, w.a.grec, qa.two, st, v2A ? A : nullptr, w.a.rec_mm,
                            w.a.grec_mm))) {
    return rc;
  }
  ag = a;
  if (!owner && qa.two && (rc = run_grad_pass(K, CAFEQ_AXIS_COL, A, 1, qa, w.a, kLossLse, 0.f, lse_t, w.hdrA, int(pa.nslot),
                                              w.member_ref, &ag, st)))
    return rc;
  if (!pair_launch && (rc = run_core(K, CAFEQ_AXIS_ROW, gb, b, w.b.rec, w.b.grec, qb.two, st, v2B ? B : nullptr, w.b.rec_mm,
                                     w.b.grec_mm)))
    return rc;
  bg = b;
  if (!owner && qb.two && (rc = run_grad_pass(K, CAFEQ_AXIS_ROW, B, x->rep, qb, w.b, kLossLse, 0.f, lse_t, w.hdrB, int(pb.nslot),
                                              w.member_ref + 1, &bg, st)))
    return rc;

  const int64_t ngroups = A->rows * (A->cols / ga.G) + (B->rows / gb.G) * B->cols;
  if (!owner && (rc = launch_reduce_losses(kLossLse, w.hdrA, int(pa.nslot), w.hdrB, int(pb.nslot), 0.f, lse_t, ngroups,
                                           losses, w.lse_ms, st)))
    return rc;
  if (grad && owner) {
    // both members' gradient passes in one launch: one workgroup per block writes member A's share into gradT
    // (transposed) and member B's G_P; d/dT = -P^T G_P P^T follows.  The pair's LogSumExp has to be known to
    // them: every workgroup reduces the partial headers itself, the first also writes the losses.
    const GradOwnerJob jobs[2] = {grad_owner_job(A, CAFEQ_AXIS_COL, qa, w.a, gradT, 1),
                                  grad_owner_job(B, CAFEQ_AXIS_ROW, qb, w.b, w.gp, 0)};
    LossArgs la{};
    la.hdrA = w.hdrA; la.nslotA = int(pa.nslot); la.hdrB = w.hdrB; la.nslotB = int(pb.nslot); la.kind = kLossLse;
    la.t = lse_t; la.ngroups = ngroups; la.losses = losses; la.lse_ms = w.lse_ms;
    if ((rc = launch_grad_owner_timed(jobs, 2, kLossLse, 0.f, lse_t, w.lse_ms, st, &la))) return rc;
    if ((rc = launch_bgemm_chain(x->Tinv, w.gp, w.x1, gradT, K, nb, -1.f, 1.f, st, adam))) return rc;
  } else if (grad) {
    // member A into gradT; member B: G_P of transform block b sums its rep row-blocks; d/dT = -P^T G_P P^T
    if ((rc = launch_reduce_grad_pair(ag, ga.Gk, qa.fused, qa.two ? w.member_ref : nullptr, gradT, bg, gb.Gk, qb.fused,
                                      qb.two ? w.member_ref + 1 : nullptr, w.gp, K, nb, w.lse_ms, st)))
      return rc;
    if ((rc = launch_bgemm_chain(x->Tinv, w.gp, w.x1, gradT, K, nb, -1.f, 1.f, st, adam))) return rc;
  }
  return CAFEQ_OK;
}

int cafeq_dual_proxy_loss_fwd_bwd(const cafeq_mat* A, const cafeq_mat* B, const cafeq_xform* x,
                                  const cafeq_quant_cfg* cfg, float lse_t, float* losses, float* gradT,
                                  int8_t* codesU, float* scalesU, int8_t* codesV, float* scalesV,
                                  void* ws, void* stream) {
  return dual_impl(A, B, x, cfg, lse_t, losses, gradT, codesU, scalesU, codesV, scalesV, ws, stream, nullptr);
}

int cafeq_adaptive_round_step(const float* U, const float* V, int64_t rowsA, int64_t colsA, int64_t rowsB,
                              int64_t colsB, const cafeq_quant_cfg* cfg, int k, int nb, int rep, int half,
                              int8_t* codesU, float* scalesU, int8_t* codesV, float* scalesV, int* status,
                              void* ws, void* stream) {
  int rc = check_cfg(cfg, false);
  if (rc) return rc;
  if (!U || !V || !codesU || !scalesU || !codesV || !scalesV) return CAFEQ_ERR_INVALID_ARG;
  if (half < 0 || half > 2) return CAFEQ_ERR_INVALID_ARG;
  if (!supported_block(k)) return CAFEQ_ERR_UNSUPPORTED;
  if (nb <= 0 || rep <= 0 || rowsA <= 0 || colsB <= 0) return CAFEQ_ERR_BAD_SHAPE;
  if (colsA != int64_t(nb) * k || rowsB != int64_t(nb) * rep * k || colsB % 4 != 0) return CAFEQ_ERR_BAD_SHAPE;
  if (!aligned16(U) || !aligned16(V) || !aligned16(codesU) || !aligned16(codesV) || !aligned16(scalesU) ||
      !aligned16(scalesV))
    return CAFEQ_ERR_BAD_ALIGN;
  if (!ws) return CAFEQ_ERR_WORKSPACE;
  AdaptivePlan ap;
  if ((rc = plan_adaptive(cfg, k, nb, rep, rowsA, colsA, rowsB, colsB, &ap))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const AdaptiveWs w = carve_adaptive(ws, ap, k, nb, nullptr);
  const QGrid grid = make_grid(cfg->bits);

  if (half == 0 || half == 1) {
    // line 3: C = pinv(Uq_b) U_b per head, Vq <- Q(C V_q)
    if ((rc = launch_gram_pair(CAFEQ_AXIS_COL, U, codesU, scalesU, rowsA, colsA, k, ap.ga.G, nb, 1, ap.chunkA,
                               ap.nchunkA, w.partial, st)))
      return rc;
    if ((rc = launch_gj_solve(k, nb, ap.nchunkA, w.partial, w.work, w.Sinv, w.Rsum, w.Cmat, status, 2, 0, st))) return rc;
    cafeq_mat mv{V, rowsB, colsB, colsB, CAFEQ_F32};
    CoreParams p;
    fill_common(&p, &mv, ap.planV, rep);
    if ((rc = launch_split_planes(w.Cmat, k, nb, 0, kFwdPlanes, w.planes, st))) return rc;
    p.Afwd = w.planes; p.Ainv = nullptr;
    p.grid = grid; p.codes = codesV; p.scales = scalesV;
    if ((rc = run_core(k, CAFEQ_AXIS_ROW, ap.gb, p, w.rec, w.grec, false, st))) return rc;
  }
  if (half == 0 || half == 2) {
    // line 4: C^T = V_[b] pinv(Vq_[b]) per head, Uq_b <- Q(U_b C^T)
    if ((rc = launch_gram_pair(CAFEQ_AXIS_ROW, V, codesV, scalesV, rowsB, colsB, k, ap.gb.G, nb, rep, ap.chunkB,
                               ap.nchunkB, w.partial, st)))
      return rc;
    if ((rc = launch_gj_solve(k, nb, rep * ap.nchunkB, w.partial, w.work, w.Sinv, w.Rsum, w.Cmat, status, 2, 1, st))) return rc;
    cafeq_mat mu{U, rowsA, colsA, colsA, CAFEQ_F32};
    CoreParams p;
    fill_common(&p, &mu, ap.planU, 1);
    if ((rc = launch_split_planes(w.Cmat, k, nb, 0, kFwdPlanes, w.planes, st))) return rc;
    p.Afwd = w.planes; p.Ainv = nullptr;
    p.grid = grid; p.codes = codesU; p.scales = scalesU;
    if ((rc = run_core(k, CAFEQ_AXIS_COL, ap.ga, p, w.rec, w.grec, false, st))) return rc;
  }
  return CAFEQ_OK;
}

}  // extern "C"
